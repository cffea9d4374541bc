// CPU build of the decode library (tests only).  The library's source is compiled as it is, against the
// stand-in <hip/hip_runtime.h> of this directory; this program reads a problem from a file, calls the
// C-ABI entry points amla_workspace_bytes and amla_decode on host buffers of exactly the documented
// sizes (AddressSanitizer sees every access past an end), and writes out and lse.
//
// input file: 12 int32 (batch, s_q, heads, num_blocks, max_blocks, variant, num_splits, flags,
//             use amla_decode_static_workspace (0/1), has q_lens (0/1), 0, 0), float softmax_scale, then q bits,
//             cache bits, block table, seqlens and, when announced, q_lens
// output file: int32 status, int32 effective splits; then, when status is 0, out bits
//             [batch * rows * 512] uint16 and lse [batch * rows] float
#include "../../paper_2509_25224_amd/csrc/amla_decode.hip"
#include "../../paper_2509_25224_amd/csrc/amla_decode_rg.hip"

namespace {
alignas(1024) uint8_t smem_raw[kRgLdsBytes > kLdsBytes ? kRgLdsBytes : kLdsBytes];   // the workgroup's dynamic LDS
}  // namespace

template <class T>
static T* alloc_exact(size_t n) {
  return static_cast<T*>(std::malloc(n ? n * sizeof(T) : 1));
}

int main(int argc, char** argv) {
  if (argc != 3) return 2;
  FILE* f = std::fopen(argv[1], "rb");
  if (!f) return 2;
  int32_t h[12];
  float scale;
  if (std::fread(h, 4, 12, f) != 12 || std::fread(&scale, 4, 1, f) != 1) return 2;
  amla_desc d;
  std::memset(&d, 0, sizeof(d));
  d.batch = h[0]; d.s_q = h[1]; d.num_heads = h[2]; d.num_blocks = h[3]; d.max_blocks_per_seq = h[4];
  d.variant = h[5]; d.num_splits = h[6]; d.flags = h[7];
  d.d_qk = kDqk; d.d_v = kDv; d.block_size = kBlock;
  const size_t n_rows = (size_t)d.batch * d.s_q * d.num_heads;
  const size_t n_kv = (size_t)d.num_blocks * kBlock * kDqk, n_tab = (size_t)d.batch * d.max_blocks_per_seq;
  // 16-byte alignment of q / cache / out is part of the entry point's contract
  uint16_t* q = static_cast<uint16_t*>(std::aligned_alloc(16, (n_rows * kDqk * 2 + 15) / 16 * 16));
  uint16_t* kv = static_cast<uint16_t*>(std::aligned_alloc(16, (n_kv * 2 + 15) / 16 * 16));
  int32_t* table = alloc_exact<int32_t>(n_tab);
  int32_t* lens = alloc_exact<int32_t>(d.batch);
  bool ok = std::fread(q, 2, n_rows * kDqk, f) == n_rows * kDqk && std::fread(kv, 2, n_kv, f) == n_kv &&
            std::fread(table, 4, n_tab, f) == n_tab && std::fread(lens, 4, d.batch, f) == (size_t)d.batch;
  int32_t* q_lens = nullptr;
  if (ok && h[9]) {
    q_lens = alloc_exact<int32_t>(d.batch);
    ok = std::fread(q_lens, 4, d.batch, f) == (size_t)d.batch;
    d.q_lens = q_lens;
  }
  std::fclose(f);
  if (!ok) return 2;
  uint16_t* out = static_cast<uint16_t*>(std::aligned_alloc(16, n_rows * kDv * 2));
  float* lse = alloc_exact<float>(n_rows);
  for (size_t i = 0; i < n_rows * kDv; ++i) out[i] = 0x7F7F;
  for (size_t i = 0; i < n_rows; ++i) lse[i] = NAN;
  const size_t ws_bytes = amla_workspace_bytes(&d);
  float* ws = static_cast<float*>(std::aligned_alloc(16, (ws_bytes + 15) / 16 * 16 + 16));
  for (size_t i = 0; i < ws_bytes / 4; ++i) ws[i] = NAN;
  d.workspace = ws_bytes ? ws : nullptr;
  d.workspace_bytes = ws_bytes;
  const int32_t splits = amla_effective_splits(&d);
  if (h[8]) {          // the entry point that brings its own workspace must not look at the caller's
    d.workspace = nullptr;
    d.workspace_bytes = 0;
  }
  const int32_t status = h[8] ? amla_decode_static_workspace(q, kv, table, lens, scale, out, lse, &d)
                              : amla_decode(q, kv, table, lens, scale, out, lse, &d);
  f = std::fopen(argv[2], "wb");
  if (!f) return 2;
  std::fwrite(&status, 4, 1, f);
  std::fwrite(&splits, 4, 1, f);
  if (status == AMLA_OK) {
    std::fwrite(out, 2, n_rows * kDv, f);
    std::fwrite(lse, 4, n_rows, f);
  }
  std::fclose(f);
  std::free(q); std::free(kv); std::free(table); std::free(lens); std::free(out); std::free(lse); std::free(ws); std::free(q_lens);
  return 0;
}
