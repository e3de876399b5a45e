"""Host-side sanitizer builds (CPU only): the oracle's C source under AddressSanitizer + UndefinedBehaviorSanitizer
on a small model (every code path of the forward pass: both sublayer kinds, skips, grouped-query heads, bf16 and
fp32 storage, the range errors), and the host half of the library's C ABI (argument checks that return before any
device call) in a library compiled with the sanitizers on its host code only."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

ORACLE_DRIVER = r'''
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
typedef struct { int32_t n_blocks, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab, max_seq; double rope_base, rms_eps;
                 int32_t weight_dtype, kv_dtype; } orc_cfg;
typedef struct orc_model orc_model;
orc_model *orc_create(const orc_cfg *, const void *, const void *, const float *, const float **, const void **, const void **,
                      const void **, const void **, const float **, const void **, const void **, const void **);
void orc_destroy(orc_model *);
int orc_forward(orc_model *, const int32_t *, int, int, const uint8_t *, int, float *, float *);
int orc_read_kv(const orc_model *, int, int, float *, float *);
static uint32_t rs = 12345u;
static float rnd(void) { rs = rs * 1664525u + 1013904223u; return ((float)(rs >> 8) / 8388608.0f - 1.0f) * 0.05f; }
static void *mat(int dtype, size_t n) {
    if (dtype == 0) { float *p = malloc(n * 4); for (size_t i = 0; i < n; ++i) p[i] = rnd(); return p; }
    uint16_t *p = malloc(n * 2);
    for (size_t i = 0; i < n; ++i) { float f = rnd(); uint32_t u; memcpy(&u, &f, 4); p[i] = (uint16_t)(u >> 16); }
    return p;
}
int main(void) {
    for (int variant = 0; variant < 2; ++variant) {
        orc_cfg c = {2, 32, 4, variant ? 2 : 4, 8, 48, 50, 12, 10000.0, 1e-5, variant, variant};
        int nb = c.n_blocks, d = c.d_model, qd = c.n_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim, F = c.d_ffn;
        void *embed = mat(c.weight_dtype, (size_t)c.vocab * d), *head = mat(c.weight_dtype, (size_t)c.vocab * d);
        float *fn = malloc(d * 4); for (int i = 0; i < d; ++i) fn[i] = 1.0f + rnd();
        const float *an[2], *mn[2]; const void *wq[2], *wk[2], *wv[2], *wo[2], *wg[2], *wu[2], *wd[2];
        for (int b = 0; b < nb; ++b) {
            float *a = malloc(d * 4), *m = malloc(d * 4);
            for (int i = 0; i < d; ++i) { a[i] = 1.0f + rnd(); m[i] = 1.0f + rnd(); }
            an[b] = a; mn[b] = m;
            wq[b] = mat(c.weight_dtype, (size_t)qd * d); wk[b] = mat(c.weight_dtype, (size_t)kvd * d);
            wv[b] = mat(c.weight_dtype, (size_t)kvd * d); wo[b] = mat(c.weight_dtype, (size_t)d * qd);
            wg[b] = mat(c.weight_dtype, (size_t)F * d); wu[b] = mat(c.weight_dtype, (size_t)F * d);
            wd[b] = mat(c.weight_dtype, (size_t)d * F);
        }
        orc_model *m = orc_create(&c, embed, head, fn, an, wq, wk, wv, wo, mn, wg, wu, wd);
        int32_t toks[12] = {1, 7, 49, 0, 3, 3, 12, 48, 5, 9, 11, 2};
        float *logits = malloc((size_t)12 * c.vocab * 4), *hidden = malloc((size_t)12 * d * 4);
        if (orc_forward(m, toks, 5, 0, NULL, 0, logits, hidden) != 0) return 1;            /* prompt */
        uint8_t mask[4] = {0, 1, 1, 0};
        if (orc_forward(m, toks + 5, 1, 5, mask, 0, logits, NULL) != 0) return 2;          /* draft step with skips */
        if (orc_forward(m, toks + 5, 7, 5, NULL, 6, logits, hidden) != 0) return 3;        /* verification up to the last slot */
        if (orc_forward(m, toks, 1, 12, NULL, 0, logits, NULL) != -1) return 4;            /* past the cache */
        if (orc_forward(m, toks, 13, 0, NULL, 0, logits, NULL) != -1) return 5;
        int32_t bad = c.vocab;
        if (orc_forward(m, &bad, 1, 0, NULL, 0, logits, NULL) != -1) return 6;
        float *k = malloc(kvd * 4), *v = malloc(kvd * 4);
        if (orc_read_kv(m, 1, 11, k, v) != 0 || orc_read_kv(m, 2, 0, k, v) != -1 || orc_read_kv(m, 0, 12, k, v) != -1) return 7;
        for (int i = 0; i < c.vocab; ++i) if (!isfinite(logits[i])) return 8;
        orc_destroy(m);
        free(k); free(v); free(logits); free(hidden); free(embed); free(head); free(fn);
        for (int b = 0; b < nb; ++b) {
            free((void *)an[b]); free((void *)mn[b]); free((void *)wq[b]); free((void *)wk[b]); free((void *)wv[b]);
            free((void *)wo[b]); free((void *)wg[b]); free((void *)wu[b]); free((void *)wd[b]);
        }
    }
    puts("oracle sanitizer run ok");
    return 0;
}
'''


def test_oracle_forward_under_asan_and_ubsan(tmp_path):
    drv = tmp_path / "driver.c"
    drv.write_text(ORACLE_DRIVER)
    exe = tmp_path / "orc_san"
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-o", str(exe), str(drv), os.path.join(ROOT, "oracle", "forward.c"), "-lm"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.returncode, r.stdout[-1000:], r.stderr[-3000:])
    assert "oracle sanitizer run ok" in r.stdout


ABI_DRIVER = r'''
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include "knnssd.h"
#define CHECK(expr, want) do { long got_ = (long)(expr); if (got_ != (long)(want)) { printf("line %d: %s = %ld, want %ld\n", __LINE__, #expr, got_, (long)(want)); return 1; } } while (0)
int main(void) {
    knnssd_model_cfg c;
    memset(&c, 0, sizeof c);
    c.n_blocks = 2; c.d_model = 256; c.n_heads = 4; c.n_kv_heads = 4; c.head_dim = 64; c.d_ffn = 704; c.vocab = 1000;
    c.max_seq = 96; c.max_anchors = 8; c.rope_base = 10000.f; c.rms_eps = 1e-5f; c.weight_dtype = KNNSSD_BF16; c.kv_dtype = KNNSSD_BF16;
    CHECK(knnssd_workspace_bytes(NULL), 0);
    CHECK(knnssd_workspace_bytes(&c) > 0, 1);
    CHECK(knnssd_kvcache_bytes(&c), (size_t)2 * 2 * 4 * 96 * 64 * 2);
    CHECK(knnssd_pack_supported(&c), 1);
    knnssd_model_cfg bad = c; bad.head_dim = 48;
    CHECK(knnssd_workspace_bytes(&bad), 0);
    bad = c; bad.prefill_mode = 7;
    CHECK(knnssd_workspace_bytes(&bad), 0);
    bad = c; bad.verify_attn = -1;
    CHECK(knnssd_workspace_bytes(&bad), 0);
    bad = c; bad.attn_merge = 2;
    CHECK(knnssd_workspace_bytes(&bad), 0);
    knnssd_ctx *h = (knnssd_ctx *)1;
    knnssd_weights w;
    memset(&w, 0, sizeof w);
    CHECK(knnssd_create(&c, &w, NULL, 0, NULL, 0, NULL, &h), KNNSSD_EINVAL);
    CHECK(h == NULL, 1);
    CHECK(knnssd_create(&c, &w, (void *)0x100000, 1, (void *)0x100000, 1, NULL, &h), KNNSSD_EINVAL);   /* buffers too small */
    CHECK(knnssd_create(NULL, NULL, NULL, 0, NULL, 0, NULL, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_destroy(NULL), KNNSSD_EINVAL);
    CHECK(knnssd_set_skipset(NULL, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_set_anchors(NULL, NULL, 0, NULL, 1, 256, NULL, 1, 4), KNNSSD_EINVAL);
    CHECK(knnssd_prefill(NULL, NULL, 0, NULL, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_select_skipset(NULL, NULL, NULL, NULL, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_knn_topk(NULL, NULL, 1, 1, NULL, NULL, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_last_selection(NULL, NULL, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_draft_step(NULL, 0, 0, NULL, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_verify(NULL, NULL, 0, 0, NULL, NULL, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_generate(NULL, NULL, 0, NULL, NULL, NULL, NULL, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_profile_pass(NULL, 0, NULL, 0, 0, NULL, NULL, NULL, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_get_logits(NULL, 0, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_read_kv(NULL, 0, 0, NULL, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_pack_matrix(&c, 9, (void *)0x100000, (void *)0x200000, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_pack_matrix(&c, 0, (void *)0x100000, (void *)0x100000, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_route_static(NULL, NULL, NULL, 1, 256, NULL, NULL), KNNSSD_EINVAL);
    CHECK(knnssd_route_static((void *)0x100000, (void *)0x100000, (void *)0x100000, 70000, 256, NULL, (void *)0x100000), KNNSSD_ERANGE);
    CHECK(knnssd_route_static((void *)0x100000, (void *)0x100000, (void *)0x100000, 8, 30, NULL, (void *)0x100000), KNNSSD_ESHAPE);
    CHECK(strcmp(knnssd_strerror(KNNSSD_OK), "ok"), 0);
    CHECK(knnssd_strerror(-99) != NULL, 1);
    puts("abi sanitizer run ok");
    return 0;
}
'''


@pytest.mark.timeout(900)
def test_abi_argument_checks_under_host_sanitizers(tmp_path):
    """The library's host code compiled with AddressSanitizer + UndefinedBehaviorSanitizer (host pass only; the device
    code is the ordinary gfx950 build), driven from plain C through every entry point's refusal path."""
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not on PATH")
    lib = tmp_path / "libknnssd_san.so"
    src = os.path.join(ROOT, "paper_2505_16162_amd", "csrc", "knnssd.hip")
    cmd = ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-o", str(lib), src]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=800)
    assert r.returncode == 0, r.stderr[-3000:]
    drv = tmp_path / "abi_driver.c"
    drv.write_text(ABI_DRIVER)
    exe = tmp_path / "abi_san"
    r = subprocess.run(["/opt/rocm/llvm/bin/clang", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                        "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(drv), str(lib),
                        "-Wl,-rpath," + str(tmp_path)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:protect_shadow_gap=0:verify_asan_link_order=0")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.returncode, r.stdout[-1500:], r.stderr[-3000:])
    assert "abi sanitizer run ok" in r.stdout
