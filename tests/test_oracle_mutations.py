"""The pins must notice a plausible mistake anywhere in the oracle: each mutant below is the
oracle with one such mistake planted (on the CPU, in a temporary copy), and the pin tests are
required to fail on it."""
import os
import subprocess
import sys

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_fp16.py", "tests/test_oracle_layout.py", "tests/test_oracle_pack_overflow.py",
             "tests/test_oracle_adam.py", "tests/test_oracle_planner.py"]

MUTANTS = [
    ("momentum sign", "m = a + b;", "m = a - b;"),
    ("variance uses g instead of g^2", "float e = d * g;", "float e = d;"),
    ("epsilon dropped", "den = den + eps;", "den = den + 0.0f;"),
    ("no bias correction of v", "float den = r * s.c2;", "float den = r;"),
    ("no bias correction of m", "s->step_size = (float)(h->lr / (1.0 - b1t));", "s->step_size = (float)(h->lr);"),
    ("update sign", "p = p - u;", "p = p + u;"),
    ("L2 decay sign", "g = g + t;", "g = g - t;"),
    ("decoupled decay dropped", "p = p * s.decay;", "p = p * 1.0f;"),
    ("no unscale", "orc_f16_to_f32(g16[k]) * s.inv_scale;", "orc_f16_to_f32(g16[k]);"),
    ("betas swapped", "float a = beta1 * m;", "float a = beta2 * m;"),
    ("no square root", "float r = sqrtf(v);", "float r = v;"),
    ("1-beta2 taken as 1-beta1", "s->omb2 = (float)(1.0 - h->beta2);", "s->omb2 = (float)(1.0 - h->beta1);"),
    ("epsilon inside the root", "float r = sqrtf(v);", "float r = sqrtf(v + eps * eps);"),
    ("layout: tensor that exactly fits opens a new chunk", "if (s > chunk_elems - cur) {", "if (s >= chunk_elems - cur) {"),
    ("layout: oversized tensor shares a started chunk", "if (cur > 0) {", "if (0) {"),
    ("overflow: nan not flagged", "if ((g16_chunks[c][k] & 0x7C00u) == 0x7C00u) f = 1;",
     "if ((g16_chunks[c][k] & 0x7FFFu) == 0x7C00u) f = 1;"),
    ("overflow: last used element missed", "for (uint64_t k = 0; k < used[c]; k++)\n            if ((g16",
     "for (uint64_t k = 0; k + 1 < used[c]; k++)\n            if ((g16"),
    ("fp16 ties round half up", "if (rem > 0x1000u || (rem == 0x1000u && (keep & 1u)))", "if (rem >= 0x1000u)"),
    ("fp16 subnormals flushed", "if (a < 0x33000000u)", "if (a < 0x38800000u)"),
    ("fp16->fp32 subnormal exponent off by one", "bits = sign | ((uint32_t)(112 - e) << 23)", "bits = sign | ((uint32_t)(113 - e) << 23)"),
    ("overflow step still updates", "        if (!flag)\n            orc_adam_chunk", "        if (1)\n            orc_adam_chunk"),
    ("skipped step leaves grads in the reused chunk", "else if (g16[c] == p16[c])", "else if (0)"),
    ("pack writes one element late", "+ (lin % chunk_elems) * elem_size;\n            for (uint64_t b = 0; b < elem_size; b++) dst[b]",
     "+ ((lin + 1) % chunk_elems) * elem_size;\n            for (uint64_t b = 0; b < elem_size; b++) dst[b]"),
    ("unpack reads one element late", "+ (lin % chunk_elems) * elem_size;\n            for (uint64_t b = 0; b < elem_size; b++) dst[k * elem_size + b]",
     "+ ((lin + 1) % chunk_elems) * elem_size;\n            for (uint64_t b = 0; b < elem_size; b++) dst[k * elem_size + b]"),
    ("re-cast misses the last element", "for (uint64_t k = 0; k < used; k++) p16[k] = orc_f32_to_f16(p32[k]);",
     "for (uint64_t k = 0; k + 1 < used; k++) p16[k] = orc_f32_to_f16(p32[k]);"),
    ("re-cast truncates instead of rounding", "for (uint64_t k = 0; k < used; k++) p16[k] = orc_f32_to_f16(p32[k]);",
     "for (uint64_t k = 0; k < used; k++) { uint32_t x; memcpy(&x, &p32[k], 4); x &= 0xFFFFE000u; float f; memcpy(&f, &x, 4); p16[k] = orc_f32_to_f16(f); }"),
    ("bias correction of v without the root", "s->c2 = (float)(1.0 / sqrt(1.0 - b2t));", "s->c2 = (float)(1.0 / (1.0 - b2t));"),
    ("unscale multiplies by the loss scale", "s->inv_scale = (float)(1.0 / h->loss_scale);", "s->inv_scale = (float)(h->loss_scale);"),
    ("beta^t with one factor too few", "for (uint64_t i = 0; i < h->step; i++) { b1t", "for (uint64_t i = 1; i < h->step; i++) { b1t"),
    ("decoupled decay factor without lr", "s->decay = (float)(1.0 - h->lr * h->weight_decay);", "s->decay = (float)(1.0 - h->weight_decay);"),
    ("scaler: t advances on an overflow step", "        s->scale = half < 1.0f ? 1.0f : half;\n        s->good_steps = 0;",
     "        s->scale = half < 1.0f ? 1.0f : half;\n        s->good_steps = 0; s->step += 1;"),
    ("scaler: scale doubles on overflow", "float half = s->scale * 0.5f;", "float half = s->scale * 2.0f;"),
    ("scaler: no floor at 1", "s->scale = half < 1.0f ? 1.0f : half;", "s->scale = half;"),
    ("scaler: good steps not reset on overflow", "        s->scale = half < 1.0f ? 1.0f : half;\n        s->good_steps = 0;",
     "        s->scale = half < 1.0f ? 1.0f : half;"),
    ("placement: only the inbound direction is charged", "if (!after) cost += 12 * used[k];", "if (0) cost += 12 * used[k];"),
    ("placement: only the outbound direction is charged", "if (!before) cost += 12 * used[k];", "if (0) cost += 12 * used[k];"),
    ("placement: budget tested on the state before the step", "resident += (uint64_t)after;", "resident += (uint64_t)before;"),
    ("placement: 4 bytes per element instead of 12", "if (!before) cost += 12 * used[k];", "if (!before) cost += 4 * used[k];"),
    ("placement: first step takes everything as resident", "int before = t == 0 ? start[k] :", "int before = t == 0 ? 1 :"),
    ("placement: budget may be exceeded by one", "if (resident > budget[t]) ok = 0;", "if (resident > budget[t] + 1) ok = 0;"),
]


def test_mutant_list_is_in_sync_with_the_source():
    src = open(os.path.join(ROOT, "oracle", "psx_oracle.c")).read()
    for name, old, new in MUTANTS:
        assert src.count(old) == 1, f"mutant '{name}': pattern occurs {src.count(old)} times"


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new):
    src = open(os.path.join(ROOT, "oracle", "psx_oracle.c")).read()
    assert src.count(old) == 1
    c = tmp_path / "mutant.c"
    so = tmp_path / "libmutant.so"
    c.write_text(src.replace(old, new))
    subprocess.check_call(["gcc", *oracle.CFLAGS, "-Wno-unused-variable", "-o", str(so), str(c), "-lm"])
    env = dict(os.environ, PSX_ORACLE_LIB=str(so))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PIN_FILES],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 1, f"the pins did not notice: {name}\n{r.stdout[-800:]}"
