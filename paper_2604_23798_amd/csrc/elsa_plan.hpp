// Host-side launch planning of libelsa: which tile shape and how many key chunks a small dense problem
// gets.  Plain C++ (no HIP): the library compiles it, and a CPU test builds the same file under
// AddressSanitizer / UBSan and sweeps it over random shapes.
#pragma once
#include <cstddef>

namespace elsa {
namespace plan {

constexpr int kCus = 256;            // compute units of the part the step times below were measured on
constexpr int kMaxSplits = 65535;

struct TileChoice { int variant, splits; };

// Bytes of FP32 workspace for the chunk states of C key chunks: part_m | part_S | part_W, each part
// 256-byte aligned.  0 for sizes the library does not serve.
size_t workspace_bytes(int B, int H, int n, int d, int num_splits);

// Tile shape (variant id of the FP32 or FP16 matrix-core family) and number of key chunks for a
// small dense problem of BH heads, n queries against nk keys, head dimension d; at most max_splits
// chunks.  The launch is played through on the host (see elsa_plan.cpp).
TileChoice choose_tiles(bool fp16_tiles, long long BH, int n, int nk, int d, int causal, int max_splits);

// The same when the values have a width of their own (d_v != d): variant 1 = 128 query rows,
// 3 = the waves of a block split the keys.
TileChoice choose_tiles_dv(bool fp16_tiles, long long BH, int n, int nk, int d, int dv, int causal, int max_splits);

// Number of key chunks when a workspace of ws_bytes is available and the caller did not ask for a
// count (requested <= 0) -- or the requested count, clamped to what the keys and the workspace allow.
int auto_splits(int requested, int B, int H, int n, int nk, int d, bool fp16_tiles, size_t ws_bytes);

// FP16 tiles at d >= 96: does the 256-row tile of eight query waves (one block per CU, the K/V tiles staged once for
// twice the rows) beat the 128-row tile of four?  Measured rule, see elsa_plan.cpp.
bool wide_fp16_tile_pays(long long BH, int n, int d, int causal);

}  // namespace plan
}  // namespace elsa
