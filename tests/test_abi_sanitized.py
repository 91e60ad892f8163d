"""The host side of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU).

Every source of the library is compiled once more with the host pass instrumented
(``-Xarch_host -fsanitize=address`` / ``undefined``; the device code is built as usual and never runs
here) and linked with a small driver that walks the argument validation, the workspace planning and
the host arithmetic of every entry point: NULL and misaligned pointers, impossible shapes, budgets out
of range, workspaces that are too small, and the sizes the planners return for the benchmark's shapes.
Validation returns before the first HIP call, so none of this needs a device.  A sanitizer report
aborts the driver; a wrong status code makes it exit non-zero.
"""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2502_14051_amd import build as libbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r"""
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include "rocketkv.h"
static int checks = 0, bad = 0;
#define EXPECT(call, want)                                                                          \
  do {                                                                                              \
    const int got_ = (int)(call);                                                                   \
    ++checks;                                                                                       \
    if (got_ != (want)) { ++bad; printf("line %d: %s -> %d (%s), expected %d\n", __LINE__, #call, got_, rocketkv_last_error(), (int)(want)); } \
  } while (0)
int main() {
  // device pointers are never dereferenced on the host: any aligned non-null value will do
  alignas(256) static unsigned char fake[4096];
  void* p = fake;
  int32_t* ip = reinterpret_cast<int32_t*>(fake);
  rocketkv_cache_t c;
  memset(&c, 0, sizeof c);
  c.batch = 16; c.n_q_heads = 32; c.n_kv_heads = 8; c.head_dim = 128; c.page_size = 16; c.pages_cap = 264;
  c.n_phys_pages = 16 * 264; c.stride_head = 16 * 128; c.stride_page = 8 * 16 * 128;
  c.seq_lens = ip; c.block_table = nullptr; c.k_pool = p; c.v_pool = p; c.v_layout = ROCKETKV_V_CHANNEL_MAJOR;
  const size_t ws = rocketkv_workspace_bytes(ROCKETKV_OP_HSA_DECODE, &c, 1024, 0);
  EXPECT(ws > ROCKETKV_WS_HEADER_BYTES && ws <= ROCKETKV_NOALLOC_SCRATCH_BYTES, 1);
  EXPECT(rocketkv_workspace_bytes(ROCKETKV_OP_HSA_DECODE, nullptr, 1024, 0), 0);
  EXPECT(rocketkv_workspace_bytes(ROCKETKV_OP_HSA_DECODE, &c, 0, 0), 0);
  EXPECT(rocketkv_workspace_bytes(99, &c, 1, 0), 0);
  EXPECT(rocketkv_workspace_bytes(ROCKETKV_OP_SNAPKV, &c, 32, 16), 0);
  EXPECT(rocketkv_workspace_bytes(ROCKETKV_OP_DENSE_DECODE, &c, 0, 0) > 0, 1);
  EXPECT(rocketkv_workspace_bytes(ROCKETKV_OP_ATTEND, &c, 64, 0) > 0, 1);
  EXPECT(rocketkv_workspace_bytes(ROCKETKV_OP_SNAPKV, &c, 32, 4096) > 0, 1);
  // decode: every refusal comes before a launch
  EXPECT(rocketkv_hsa_decode(nullptr, p, p, p, 32, 1024, 0, p, nullptr, nullptr, nullptr, p, ws, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_hsa_decode(&c, nullptr, p, p, 32, 1024, 0, p, nullptr, nullptr, nullptr, p, ws, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_hsa_decode(&c, p, p, p, 0, 1024, 0, p, nullptr, nullptr, nullptr, p, ws, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_hsa_decode(&c, p, p, p, 129, 1024, 0, p, nullptr, nullptr, nullptr, p, ws, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_hsa_decode(&c, p, p, p, 32, 0, 0, p, nullptr, nullptr, nullptr, p, ws, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_hsa_decode(&c, p, p, p, 32, 1024, -1, p, nullptr, nullptr, nullptr, p, ws, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_hsa_decode(&c, p, p, p, 32, 1024, 0, nullptr, nullptr, nullptr, nullptr, p, ws, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_hsa_decode(&c, p, p, p, 32, 1024, 0, p, nullptr, nullptr, nullptr, p, ws - 1, nullptr), ROCKETKV_WORKSPACE_TOO_SMALL);
  EXPECT(rocketkv_hsa_decode(&c, p, p, p, 32, 1024, 0, p, nullptr, nullptr, nullptr, nullptr, ws, nullptr), ROCKETKV_WORKSPACE_TOO_SMALL);
  EXPECT(rocketkv_hsa_decode(&c, p, p, p, 32, 1024, 0, p, nullptr, nullptr, nullptr, fake + 16, ws, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_hsa_decode(&c, fake + 2, p, p, 32, 1024, 0, p, nullptr, nullptr, nullptr, p, ws, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_hsa_decode_append(&c, p, nullptr, p, p, p, 32, 1024, 0, p, nullptr, nullptr, nullptr, p, ws, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_hsa_decode_noalloc(nullptr, p, p, p, 32, 1024, 0, p, nullptr, nullptr, nullptr, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_hsa_decode_noalloc(&c, p, p, p, 32, 0, 0, p, nullptr, nullptr, nullptr, nullptr), ROCKETKV_INVALID_ARG);
  {
    rocketkv_cache_t big = c;  // scratch need beyond the built-in buffer: refused, nothing looked up or launched
    big.batch = 128; big.pages_cap = 1032; big.n_phys_pages = 128 * 1032;
    EXPECT(rocketkv_workspace_bytes(ROCKETKV_OP_HSA_DECODE, &big, 1024, 0) > ROCKETKV_NOALLOC_SCRATCH_BYTES, 1);
    EXPECT(rocketkv_hsa_decode_noalloc(&big, p, p, p, 32, 1024, 0, p, nullptr, nullptr, nullptr, nullptr), ROCKETKV_UNSUPPORTED);
  }
  // shapes
  {
    rocketkv_cache_t d = c; d.head_dim = 64;
    EXPECT(rocketkv_build_page_summaries(&d, p, p, 0, -1, nullptr), ROCKETKV_UNSUPPORTED);
    d = c; d.n_q_heads = 30;
    EXPECT(rocketkv_build_page_summaries(&d, p, p, 0, -1, nullptr), ROCKETKV_INVALID_ARG);
    d = c; d.n_q_heads = 8 * 32;
    EXPECT(rocketkv_build_page_summaries(&d, p, p, 0, -1, nullptr), ROCKETKV_UNSUPPORTED);
    d = c; d.pages_cap = 260;
    EXPECT(rocketkv_build_page_summaries(&d, p, p, 0, -1, nullptr), ROCKETKV_INVALID_ARG);
    d = c; d.page_size = 0;
    EXPECT(rocketkv_build_page_summaries(&d, p, p, 0, -1, nullptr), ROCKETKV_INVALID_ARG);
    d = c; d.page_size = 65;
    EXPECT(rocketkv_build_page_summaries(&d, p, p, 0, -1, nullptr), ROCKETKV_UNSUPPORTED);
    d = c; d.n_phys_pages = 10;
    EXPECT(rocketkv_build_page_summaries(&d, p, p, 0, -1, nullptr), ROCKETKV_INVALID_ARG);
    d = c; d.n_phys_pages = (int64_t)1 << 31;
    EXPECT(rocketkv_build_page_summaries(&d, p, p, 0, -1, nullptr), ROCKETKV_UNSUPPORTED);
    d = c; d.stride_head = 100;
    EXPECT(rocketkv_build_page_summaries(&d, p, p, 0, -1, nullptr), ROCKETKV_INVALID_ARG);
    d = c; d.v_layout = 7;
    EXPECT(rocketkv_build_page_summaries(&d, p, p, 0, -1, nullptr), ROCKETKV_INVALID_ARG);
    d = c; d.k_pool = nullptr;
    EXPECT(rocketkv_build_page_summaries(&d, p, p, 0, -1, nullptr), ROCKETKV_INVALID_ARG);
    EXPECT(rocketkv_build_page_summaries(&c, nullptr, p, 0, -1, nullptr), ROCKETKV_INVALID_ARG);
    EXPECT(rocketkv_build_page_summaries(&c, p, p, 265, -1, nullptr), ROCKETKV_INVALID_ARG);
    d = c; d.page_size = 3; d.stride_head = 3 * 128 + 8 - (3 * 128) % 8; d.stride_page = 8 * d.stride_head;
    EXPECT(rocketkv_attend(&d, p, ip, 8, p, nullptr, p, 1 << 20, nullptr), ROCKETKV_UNSUPPORTED);  // channel-major V needs pages of 16
  }
  EXPECT(rocketkv_hsa_select(&c, p, p, p, 32, 1024, 0, nullptr, 64, nullptr, nullptr, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_hsa_select(&c, p, p, p, 32, 1024, 0, ip, 63, nullptr, nullptr, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_attend(&c, p, ip, 0, p, nullptr, p, 1 << 20, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_attend(&c, p, ip, 64, p, nullptr, p, 16, nullptr), ROCKETKV_WORKSPACE_TOO_SMALL);
  EXPECT(rocketkv_dense_decode(&c, p, nullptr, nullptr, p, 1 << 20, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_append_kv(&c, p, nullptr, p, p, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_workspace_init(nullptr, 100, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_workspace_init(fake + 8, 100, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_stream_read(nullptr, 16, p, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_stream_read(p, 17, p, nullptr), ROCKETKV_INVALID_ARG);
  EXPECT(rocketkv_stream_read(p, 0, p, nullptr), ROCKETKV_OK);
  // Stage 1
  {
    rocketkv_cache_t dst = c; dst.k_pool = fake + 2048; dst.v_pool = fake + 2048;
    const size_t sws = rocketkv_workspace_bytes(ROCKETKV_OP_SNAPKV, &c, 32, 2048);
    EXPECT(rocketkv_snapkv_compress(nullptr, &c, 32, 63, 2048, &dst, nullptr, p, sws, nullptr), ROCKETKV_INVALID_ARG);
    EXPECT(rocketkv_snapkv_compress(p, &c, 24, 63, 2048, &dst, nullptr, p, sws, nullptr), ROCKETKV_UNSUPPORTED);
    EXPECT(rocketkv_snapkv_compress(p, &c, 0, 63, 2048, &dst, nullptr, p, sws, nullptr), ROCKETKV_INVALID_ARG);
    EXPECT(rocketkv_snapkv_compress(p, &c, 32, 64, 2048, &dst, nullptr, p, sws, nullptr), ROCKETKV_INVALID_ARG);
    EXPECT(rocketkv_snapkv_compress(p, &c, 32, 1025, 2048, &dst, nullptr, p, sws, nullptr), ROCKETKV_UNSUPPORTED);
    EXPECT(rocketkv_snapkv_compress(p, &c, 32, 63, 32, &dst, nullptr, p, sws, nullptr), ROCKETKV_INVALID_ARG);
    EXPECT(rocketkv_snapkv_compress(p, &c, 32, 63, 2048, &c, nullptr, p, sws, nullptr), ROCKETKV_INVALID_ARG);  // same pools
    EXPECT(rocketkv_snapkv_compress(p, &c, 32, 63, 2048, &dst, nullptr, p, sws - 1, nullptr), ROCKETKV_WORKSPACE_TOO_SMALL);
    EXPECT(rocketkv_snapkv_compress(p, &c, 32, 63, 264 * 16 + 1, &dst, nullptr, p, 1u << 30, nullptr), ROCKETKV_INVALID_ARG);
    rocketkv_index_t ix = {ip, ip, 16, 264};
    EXPECT(rocketkv_snapkv_filter(p, &c, 32, 63, 2048, nullptr, p, sws, nullptr), ROCKETKV_INVALID_ARG);
    ix.pages_cap = 8;
    EXPECT(rocketkv_snapkv_filter(p, &c, 32, 63, 2048, &ix, p, sws, nullptr), ROCKETKV_INVALID_ARG);
  }
  // multi-turn: the cache behind an index needs token-major V
  {
    rocketkv_index_t ix = {ip, ip, 16, 264};
    EXPECT(rocketkv_mt_hsa_decode(&c, &ix, p, p, p, 32, 1024, 0, p, nullptr, nullptr, nullptr, p, 1 << 22, nullptr), ROCKETKV_UNSUPPORTED);
    rocketkv_cache_t t = c; t.v_layout = ROCKETKV_V_TOKEN_MAJOR;
    EXPECT(rocketkv_mt_workspace_bytes(&t, &ix, 1024) > 0, 1);
    EXPECT(rocketkv_mt_workspace_bytes(&t, nullptr, 1024), 0);
    EXPECT(rocketkv_mt_hsa_decode(&t, nullptr, p, p, p, 32, 1024, 0, p, nullptr, nullptr, nullptr, p, 1 << 22, nullptr), ROCKETKV_INVALID_ARG);
    EXPECT(rocketkv_mt_hsa_decode(&t, &ix, p, p, p, 32, 1024, 0, p, nullptr, nullptr, nullptr, p, 64, nullptr), ROCKETKV_WORKSPACE_TOO_SMALL);
    EXPECT(rocketkv_mt_append_kv(&t, &ix, nullptr, p, p, p, nullptr), ROCKETKV_INVALID_ARG);
    EXPECT(rocketkv_mt_build_page_summaries(&t, &ix, p, p, 300, -1, nullptr), ROCKETKV_INVALID_ARG);
    EXPECT(rocketkv_mt_hsa_decode_append(&t, &ix, p, nullptr, p, p, p, 32, 1024, 0, p, nullptr, nullptr, nullptr, p, 1 << 22, nullptr), ROCKETKV_INVALID_ARG);
  }
  // host arithmetic
  {
    rocketkv_split_t s;
    EXPECT(rocketkv_decompose(32768, 512, 128, &s), ROCKETKV_OK);
    EXPECT(s.page_size == 3 && s.keep_budget > 0 && s.channel_budget > 0 && s.attend_tokens == 256, 1);
    EXPECT(rocketkv_decompose(0, 512, 128, &s), ROCKETKV_INVALID_ARG);
    EXPECT(rocketkv_decompose(32768, 512, 128, nullptr), ROCKETKV_INVALID_ARG);
    EXPECT(rocketkv_decompose((int64_t)1 << 41, 512, 128, &s), ROCKETKV_INVALID_ARG);
    EXPECT(rocketkv_decompose(100, 1000, 128, &s), ROCKETKV_OK);
    EXPECT(rocketkv_version() > 0, 1);
  }
  printf("%d checks, %d wrong\n", checks, bad);
  return bad ? 1 : 0;
}
"""


def test_abi_host_side_runs_clean_under_sanitizers(tmp_path):
    hipcc = libbuild._hipcc()
    clang = os.path.join(os.path.dirname(hipcc), "..", "llvm", "bin", "clang++")
    if not os.path.exists(clang):
        pytest.skip("the ROCm clang++ that matches hipcc's sanitizer runtime is not at its usual place")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=all"]
    flags = [f for f in libbuild.FLAGS if f not in ("-O3", "-Rpass-analysis=kernel-resource-usage")] + ["-O1", "-g"]

    def one(src):
        obj = tmp_path / src.replace(".hip", ".o")
        r = subprocess.run([hipcc, *flags, *san, "-c", os.path.join(libbuild.CSRC, src), "-o", str(obj)],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        return str(obj)

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(one, libbuild.SOURCES))
    (tmp_path / "driver.cpp").write_text(DRIVER)
    subprocess.run([clang, "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-I" + os.path.join(ROOT, "include"), "-c", str(tmp_path / "driver.cpp"), "-o",
                    str(tmp_path / "driver.o")], check=True)
    exe = tmp_path / "abi_san"
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize",
                        str(tmp_path / "driver.o"), *objs, "-o", str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    # (the HIP runtime keeps a few allocations for the life of the process: leak checking is for the oracle's test)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, (r.stdout[-3000:] + "\n" + r.stderr[-3000:])
    assert " 0 wrong" in r.stdout, r.stdout
