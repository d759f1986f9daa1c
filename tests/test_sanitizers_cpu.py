"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The library's host side (test-mask generator, offline weight transform, builders of the kernels'
private layouts, accessors, block selectors) and the C oracle are compiled with gcc and -fsanitize=address,undefined
into one small driver program together with a stub for the device half of the library, and the
driver walks through packing, every layout and the error paths of the five benchmark-shaped
layers at reduced size.  Any out-of-bounds access, leak, signed overflow or misaligned access in
host code makes the driver exit non-zero."""
import os
import shutil
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2407_19644_amd", "csrc")

DRIVER = r"""
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#include "ubp_internal.h"

extern "C" {
int ubp_oracle_validate(int32_t M, int32_t K, int32_t bh, int32_t bw, const int32_t *blocks, int64_t nb, int64_t *kept);
int ubp_oracle_pack(const void *W, int64_t esz, int64_t ldw, int32_t M, int32_t K, int32_t bh, int32_t bw,
                    const int32_t *blocks, int64_t nb, int32_t *indptr, int32_t *indices, void *values);
}

// the device half of the library: nothing to do on a machine without a GPU
namespace ubp {
ubp_status upload(ubp_packed *) { return UBP_ERR_DEVICE; }
void release_device(ubp_packed *) {}
}

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); return 1; } } while (0)

static int one(int M, int K, int bh, int bw, double density, int mode, ubp_dtype dt) {
    int64_t nb = ubp_target_block_count(M, K, bh, bw, density);
    CHECK(nb >= 0);
    std::vector<ubp_block> blocks((size_t)nb + 1);
    int64_t got = 0;
    CHECK(ubp_select_reference(M, K, bh, bw, density, 7, mode, 1.1, blocks.data(), nb, &got) == UBP_OK && got == nb);
    int64_t kept = 0;
    CHECK(ubp_oracle_validate(M, K, bh, bw, &blocks[0].r, nb, &kept) == 0 && kept == nb * bh * bw);
    const size_t esz = dt == UBP_F32 ? 4 : 2;
    std::vector<unsigned char> W((size_t)M * K * esz);
    for (size_t i = 0; i < W.size(); ++i) W[i] = (unsigned char)(1 + i % 120);   // finite patterns in every type
    ubp_packed *p = nullptr;
    CHECK(ubp_pack(W.data(), dt, M, K, K, bh, bw, blocks.data(), nb, UBP_HOST_ONLY, &p) == UBP_OK && p);
    int64_t n1 = 0, n2 = 0, n3 = 0;
    const int32_t *indptr = ubp_packed_indptr(p, &n1);
    const int32_t *indices = ubp_packed_indices(p, &n2);
    const void *values = ubp_packed_values(p, &n3);
    CHECK(n1 == M - bh + 2 && n2 == nb && n3 == nb * bh * bw);
    std::vector<int32_t> o_ptr((size_t)n1), o_idx((size_t)nb + 1);
    std::vector<unsigned char> o_val((size_t)(n3 + 1) * esz);
    CHECK(ubp_oracle_pack(W.data(), (int64_t)esz, K, M, K, bh, bw, &blocks[0].r, nb, o_ptr.data(), o_idx.data(), o_val.data()) == 0);
    CHECK(std::memcmp(indptr, o_ptr.data(), (size_t)n1 * 4) == 0);
    CHECK(nb == 0 || std::memcmp(indices, o_idx.data(), (size_t)nb * 4) == 0);
    CHECK(n3 == 0 || std::memcmp(values, o_val.data(), (size_t)n3 * esz) == 0);
    for (int what = 0; what < 12; ++what) (void)ubp_packed_info(p, what);
    for (int what = 100; what < 109; ++what) (void)ubp_packed_info(p, what);
    for (int what = 300; what < 312; ++what) (void)ubp_packed_info(p, what);
    for (int which = 1; which <= 3; ++which)
        for (int G : {1, 2, 4, 5})
            for (int CT : {2, 4, 8}) {
                int32_t nrg = 0;
                const int32_t *a = nullptr, *b = nullptr;
                const uint32_t *s = nullptr, *m = nullptr;
                int64_t sw = 0, mw = 0;
                ubp_status rc = ubp_packed_layout(p, G, CT, which, &nrg, &a, &b, &s, &sw, &m, &mw);
                if (rc == UBP_OK && s && sw > 0) {
                    volatile uint32_t sink = s[0] ^ s[sw - 1];   // both ends are readable
                    (void)sink;
                }
            }
    // error paths
    ubp_packed *q = nullptr;
    ubp_block bad[2] = {{0, 0}, {bh > 1 ? bh - 1 : 0, 0}};
    if (M >= 2 * bh && bh > 1) CHECK(ubp_pack(W.data(), dt, M, K, K, bh, bw, bad, 2, UBP_HOST_ONLY, &q) == UBP_ERR_OVERLAP && !q);
    ubp_block out = {M - bh + 1, 0};
    CHECK(ubp_pack(W.data(), dt, M, K, K, bh, bw, &out, 1, UBP_HOST_ONLY, &q) == UBP_ERR_OUT_OF_BOUNDS && !q);
    CHECK(ubp_pack(W.data(), dt, M, K, K, bh, bw, blocks.data(), nb, 0, &q) == UBP_ERR_DEVICE && !q);   // the stub has no device
    ubp_packed_free(p);
    // block selection on the same weights (16-bit patterns read as numbers; fp32 patterns are finite too)
    if (dt != UBP_F32) {
        const int64_t b = (int64_t)M * (K / bw);
        std::vector<double> S((size_t)b);
        CHECK(ubp_block_scores(W.data(), dt, K, M, K, bh, bw, 0, S.data(), b) == UBP_OK);
        std::vector<int64_t> I((size_t)nb + 1);
        std::vector<ubp_block> chosen((size_t)nb + 1);
        for (int method = 0; method < 3; ++method) {
            int64_t count = 0;
            ubp_status rc = method == 0 ? ubp_select_greedy(S.data(), b, bh, nb, I.data(), &count)
                          : method == 1 ? ubp_select_bed(S.data(), b, bh, nb, I.data(), &count)
                                        : ubp_select_optimal(S.data(), b, bh, nb, I.data(), &count);
            CHECK(rc == UBP_OK || (method == 2 && (rc == UBP_ERR_INFEASIBLE || rc == UBP_ERR_UNSUPPORTED)));
            if (rc != UBP_OK) continue;
            CHECK(count <= nb);
            CHECK(ubp_selection_to_blocks(I.data(), count, M, bw, chosen.data()) == UBP_OK);
            ubp_packed *s = nullptr;
            CHECK(ubp_pack(W.data(), dt, M, K, K, bh, bw, chosen.data(), count, UBP_HOST_ONLY, &s) == UBP_OK);
            double eff = 0.0, l1[3];
            CHECK(ubp_selection_efficacy(W.data(), dt, K, M, K, bh, bw, chosen.data(), count, blocks.data(), nb, l1, &eff) == UBP_OK);
            ubp_packed_free(s);
        }
        int64_t got = 0;
        CHECK(ubp_select_blocks(W.data(), dt, K, M, K, bh, bw, density, 1, 1, chosen.data(), nb, &got) == UBP_OK && got <= nb);
    }
    return 0;
}

int main() {
    int rc = 0;
    rc |= one(64, 64, 4, 4, 0.5, 0, UBP_F32);
    rc |= one(240, 160, 4, 4, 0.3, 0, UBP_F16);
    rc |= one(256, 256, 8, 8, 0.2, 0, UBP_F16);
    rc |= one(128, 1152, 4, 4, 0.25, 0, UBP_BF16);
    rc |= one(512, 2048, 16, 16, 0.1, 1, UBP_BF16);
    rc |= one(70, 45, 3, 1, 0.4, 0, UBP_BF16);
    rc |= one(90, 64, 20, 3, 0.25, 0, UBP_F16);
    rc |= one(150, 1300, 16, 40, 0.2, 0, UBP_BF16);
    rc |= one(33, 15, 5, 3, 0.3, 0, UBP_F16);
    rc |= one(16, 16, 16, 16, 1.0, 0, UBP_BF16);
    rc |= one(40, 40, 4, 4, 0.0, 0, UBP_F32);
    std::printf(rc ? "FAILED\n" : "sanitized host run ok\n");
    return rc;
}
"""


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("gcc") is None, reason="needs gcc / g++")
def test_host_code_under_asan_and_ubsan(tmp_path):
    drv = tmp_path / "driver.cpp"
    drv.write_text(textwrap.dedent(DRIVER))
    exe = tmp_path / "driver"
    orc = tmp_path / "oracle.o"
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
    subprocess.check_call(["gcc", "-std=c99", "-c", os.path.join(ROOT, "oracle", "ubp_oracle.c"), "-o", str(orc)] + san)
    subprocess.check_call(["g++", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", CSRC, str(drv),
                           os.path.join(CSRC, "ubp_host.cpp"), os.path.join(CSRC, "ubp_layouts.cpp"),
                           os.path.join(CSRC, "ubp_select.cpp"), str(orc),
                           "-o", str(exe), "-static-libasan", "-static-libubsan", "-pthread"] + san)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    res = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    sys.stdout.write(res.stdout[-2000:])
    assert res.returncode == 0 and "sanitized host run ok" in res.stdout, res.stdout[-4000:]
