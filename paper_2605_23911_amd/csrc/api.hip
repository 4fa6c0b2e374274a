// C ABI of the library (include/moe.h): argument checks on the host, workspace layout, and
// the stage launchers strung together.  Nothing here allocates, copies or synchronises.
#include <cmath>

#include "moe_internal.hpp"

namespace moe {
int g_knobs[kNumKnobs] = {-1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1};
}

namespace {

using namespace moe;

constexpr size_t kAlign = 256;

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

constexpr int kTileHeights[] = {32, 64, 96, 128, 160, 192, 256};

bool valid_tile_m(int m) {
    for (int v : kTileHeights)
        if (v == m) return true;
    return false;
}

moe_status check_config(const moe_config* c) {
    if (c == nullptr) return MOE_ERR_NULL;
    if (c->T < 0 || c->d < 1 || c->F < 1 || c->E < 1 || c->k < 1 || c->k > c->E) return MOE_ERR_SHAPE;
    if (c->gating < MOE_GATE_SOFTMAX || c->gating > MOE_GATE_SIGMOID_NORM) return MOE_ERR_SHAPE;
    if ((c->flags & ~MOE_FLAG_FUSE_COMBINE) != 0) return MOE_ERR_SHAPE;
    if (c->tile_m != 0 && !valid_tile_m(c->tile_m)) return MOE_ERR_SHAPE;
    if (c->E > kMaxExperts) return MOE_ERR_UNSUPPORTED;
    if (c->d % 64 != 0 || c->F % 64 != 0) return MOE_ERR_UNSUPPORTED;
    if ((long long)c->T * c->k > (1ll << 30)) return MOE_ERR_UNSUPPORTED;
    // the GEMM kernels address activation rows with 32-bit byte offsets: x, x_perm and h stay below 4 GiB
    const unsigned long long R = (unsigned long long)c->T * c->k;
    if (R * (unsigned long long)(c->d > c->F ? c->d : c->F) * 2ull >= (1ull << 32)) return MOE_ERR_UNSUPPORTED;
    return MOE_OK;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

size_t list_bytes(const moe_config* c, int M) { return align_up((size_t)moe_max_blocks(c, M) * 2 * sizeof(int32_t)); }
// Algorithm 1's block list, the same blocks with the multi-block experts first (for the down
// projection, see permute.hip), and one 256-byte slot holding num_blocks and num_heavy.
size_t schedule_bytes(const moe_config* c, int M) { return 2 * list_bytes(c, M) + kAlign; }

size_t arrive_bytes(const moe_config* c) {
    return align_up((size_t)(c->T > 0 ? c->T : 1) * combine_groups(*c) * sizeof(int32_t));
}

size_t hist_bytes(const moe_config* c) {
    size_t n = (size_t)permute_chunks(*c) * c->E * sizeof(int32_t);
    return align_up(n ? n : 1);
}

moe_status hip_status(hipError_t e) { return e == hipSuccess ? MOE_OK : MOE_ERR_HIP; }



}  // namespace

extern "C" {

// Test hook, not declared in include/moe.h: sets one of the knobs of moe_internal.hpp and returns
// its previous value (-2 for an unknown knob).  value = -1 restores the selection rule.
int32_t moe_test_knob(int32_t which, int32_t value) {
    if (which < 0 || which >= kNumKnobs) return -2;
    const int old = g_knobs[which];
    g_knobs[which] = value;
    return old;
}

const char* moe_status_string(moe_status s) {
    switch (s) {
        case MOE_OK: return "ok";
        case MOE_ERR_NULL: return "required pointer is NULL";
        case MOE_ERR_SHAPE: return "invalid shape or option";
        case MOE_ERR_ALIGN: return "pointer is not 16-byte aligned";
        case MOE_ERR_WORKSPACE: return "workspace too small";
        case MOE_ERR_UNSUPPORTED: return "configuration outside the supported limits";
        case MOE_ERR_HIP: return "HIP launch error";
    }
    return "unknown status";
}

int32_t moe_tile_m(const moe_config* c) {
    if (check_config(c) != MOE_OK) return 0;
    if (c->tile_m != 0) return c->tile_m;
    // One tile height serves everything: Algorithm 1 runs with M = 256 and the GEMM kernel picks
    // its body per block from the rows the block really holds, so an expert of any size up to
    // 256 rows is ONE block (its weights stream once) and a heavier expert is cut into 256-row
    // blocks.  Only when the down projection would have too few workgroups to fill the chip
    // (a handful of rows in all) the schedule uses 32-row blocks for the K-split kernel.
    const long long R = (long long)c->T * c->k;
    const long long active = c->E < R ? c->E : R;
    if ((long long)(c->d / 128) * active < 256 && R <= 32) return 32;
    if (two_workgroups_per_cu(*c)) return 128;   // see moe_internal.hpp
    return 256;
}

const char* moe_ffn_kernel_name(const moe_config* c, int32_t stage, int32_t packed) {
    if (check_config(c) != MOE_OK || (stage != 0 && stage != 1)) return nullptr;
    const int M = moe_tile_m(c);
    return stage == 0 ? gate_up_variant_name(*c, M, packed != 0) : down_variant_name(*c, M, packed != 0);
}

int32_t moe_max_blocks(const moe_config* c, int32_t M) {
    if (check_config(c) != MOE_OK || M < 1 || M > (1 << 30)) return 0;
    const long long R = (long long)c->T * c->k;
    return (int32_t)(R / M + (R < c->E ? R : c->E));
}

size_t moe_route_workspace_size(const moe_config* c) {
    return check_config(c) == MOE_OK ? align_up(route_workspace_bytes(*c) + 1) : 0;
}

size_t moe_permute_workspace_size(const moe_config* c) {
    return check_config(c) == MOE_OK ? hist_bytes(c) : 0;
}

size_t moe_ffn_workspace_size(const moe_config* c) {
    return check_config(c) == MOE_OK ? schedule_bytes(c, moe_tile_m(c)) : 0;
}

moe_status moe_forward_workspace_layout(const moe_config* c, moe_workspace_layout* out) {
    const moe_status st = check_config(c);
    if (st != MOE_OK) return st;
    if (out == nullptr) return MOE_ERR_NULL;
    const size_t R = (size_t)c->T * c->k;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes ? bytes : 1); return o; };
    out->topk_idx = take(R * sizeof(int32_t));
    out->topk_w = take(R * sizeof(float));
    out->counts = take((size_t)c->E * sizeof(int32_t));
    out->offsets = take((size_t)(c->E + 1) * sizeof(int32_t));
    out->row_of = take(R * sizeof(int32_t));
    out->src_of = take(R * sizeof(int32_t));
    out->x_perm = take(0);   // moe_forward gathers rows inside the gate+up loads: no permuted copy of x
    out->h = take(R * c->F * sizeof(uint16_t));
    out->y_perm = take(R * c->d * sizeof(uint16_t));
    out->scratch = take(moe_route_workspace_size(c) + hist_bytes(c) + schedule_bytes(c, moe_tile_m(c)) + arrive_bytes(c));
    out->total = off;
    return MOE_OK;
}

size_t moe_forward_workspace_size(const moe_config* c) {
    moe_workspace_layout l;
    return moe_forward_workspace_layout(c, &l) == MOE_OK ? l.total : 0;
}

size_t moe_workspace_size(const moe_config* c) { return moe_forward_workspace_size(c); }

moe_status moe_route(const moe_config* c, const void* x, const void* W_r, const float* bias,
                     int32_t* topk_idx, float* topk_w, void* workspace, size_t ws_bytes, void* stream) {
    const moe_status st = check_config(c);
    if (st != MOE_OK) return st;
    if (!x || !W_r || !topk_idx || !topk_w || !workspace) return MOE_ERR_NULL;
    if (misaligned(x) || misaligned(W_r) || misaligned(workspace)) return MOE_ERR_ALIGN;
    if (ws_bytes < moe_route_workspace_size(c)) return MOE_ERR_WORKSPACE;
    if (c->T == 0) return MOE_OK;
    return hip_status(launch_route(*c, (const uint16_t*)x, (const uint16_t*)W_r, bias, topk_idx, topk_w, workspace,
                                   nullptr, 0, (hipStream_t)stream));
}

moe_status moe_permute(const moe_config* c, const void* x, const int32_t* topk_idx, int32_t* counts,
                       int32_t* offsets, int32_t* row_of, int32_t* src_of, void* x_perm, void* workspace,
                       size_t ws_bytes, void* stream) {
    const moe_status st = check_config(c);
    if (st != MOE_OK) return st;
    if (!topk_idx || !counts || !offsets || !row_of || !src_of || !workspace) return MOE_ERR_NULL;
    if ((x == nullptr) != (x_perm == nullptr)) return MOE_ERR_NULL;
    if (misaligned(x) || misaligned(x_perm) || misaligned(workspace)) return MOE_ERR_ALIGN;
    if (ws_bytes < moe_permute_workspace_size(c)) return MOE_ERR_WORKSPACE;
    if (c->T == 0) return MOE_OK;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = launch_permute_index(*c, topk_idx, counts, offsets, row_of, src_of, (int32_t*)workspace, 0,
                                        nullptr, nullptr, nullptr, nullptr, s);
    if (e == hipSuccess && x != nullptr && c->T > 0)
        e = launch_gather_rows(*c, (const uint16_t*)x, src_of, (uint16_t*)x_perm, c->d, s);
    return hip_status(e);
}

moe_status moe_permute_static(const moe_config* c, const void* x, const int32_t* topk_idx, int32_t* counts,
                              int32_t* offsets, int32_t* row_of, int32_t* src_of, void* x_perm, void* stream) {
    const moe_status st = check_config(c);
    if (st != MOE_OK) return st;
    if (!topk_idx || !counts || !offsets || !row_of || !src_of) return MOE_ERR_NULL;
    if ((x == nullptr) != (x_perm == nullptr)) return MOE_ERR_NULL;
    if (misaligned(x) || misaligned(x_perm)) return MOE_ERR_ALIGN;
    // the chunk histograms [chunks, E] must fit the file-scope array
    if ((size_t)permute_chunks(*c) * (size_t)c->E > (size_t)MOE_PERMUTE_STATIC_MAX_INTS) return MOE_ERR_UNSUPPORTED;
    if (c->T == 0) return MOE_OK;
    int32_t* hist = nullptr;
    hipError_t e = permute_static_scratch(&hist);
    hipStream_t s = (hipStream_t)stream;
    if (e == hipSuccess)
        e = launch_permute_index(*c, topk_idx, counts, offsets, row_of, src_of, hist, 0, nullptr, nullptr, nullptr, nullptr, s);
    if (e == hipSuccess && x != nullptr)
        e = launch_gather_rows(*c, (const uint16_t*)x, src_of, (uint16_t*)x_perm, c->d, s);
    return hip_status(e);
}

moe_status moe_block_schedule(const moe_config* c, const int32_t* offsets, int32_t M, int32_t* blocks,
                              int32_t* num_blocks, void* stream) {
    const moe_status st = check_config(c);
    if (st != MOE_OK) return st;
    if (M < 1 || M > (1 << 30)) return MOE_ERR_SHAPE;   // ceil(n_e / M) is computed as (n_e + M - 1) / M in 32 bits
    if (!offsets || !blocks || !num_blocks) return MOE_ERR_NULL;
    if (c->T == 0) return MOE_OK;
    return hip_status(launch_block_schedule(*c, offsets, M, blocks, num_blocks, nullptr, nullptr, (hipStream_t)stream));
}

size_t moe_packed_weights_size(const moe_config* c) {
    return check_config(c) == MOE_OK ? packed_gate_up_bytes(*c) + packed_down_bytes(*c) : 0;
}

moe_status moe_pack_weights(const moe_config* c, const void* W_gate, const void* W_up, const void* W_down,
                            void* packed, void* stream) {
    const moe_status st = check_config(c);
    if (st != MOE_OK) return st;
    if (!W_gate || !W_up || !W_down || !packed) return MOE_ERR_NULL;
    if (misaligned(W_gate) || misaligned(W_up) || misaligned(W_down) ||
        (reinterpret_cast<uintptr_t>(packed) & (kAlign - 1)) != 0)
        return MOE_ERR_ALIGN;
    return hip_status(launch_pack(*c, (const uint16_t*)W_gate, (const uint16_t*)W_up, (const uint16_t*)W_down,
                                  (uint16_t*)packed, (hipStream_t)stream));
}

moe_status moe_grouped_ffn(const moe_config* c, const void* x_perm, const int32_t* offsets, const void* W_gate,
                           const void* W_up, const void* W_down, const void* W_packed, void* h, void* y_perm,
                           void* workspace, size_t ws_bytes, void* stream) {
    const moe_status st = check_config(c);
    if (st != MOE_OK) return st;
    if (!x_perm || !offsets || !h || !y_perm || !workspace) return MOE_ERR_NULL;
    if (!W_packed && (!W_gate || !W_up || !W_down)) return MOE_ERR_NULL;
    if (misaligned(x_perm) || misaligned(W_gate) || misaligned(W_up) || misaligned(W_down) || misaligned(h) ||
        misaligned(y_perm) || misaligned(workspace) || (reinterpret_cast<uintptr_t>(W_packed) & (kAlign - 1)) != 0)
        return MOE_ERR_ALIGN;
    if (ws_bytes < moe_ffn_workspace_size(c)) return MOE_ERR_WORKSPACE;
    if (c->T == 0) return MOE_OK;
    hipStream_t s = (hipStream_t)stream;
    const int M = moe_tile_m(c);
    int32_t* blocks = (int32_t*)workspace;
    int32_t* blocks_mix = (int32_t*)((char*)workspace + list_bytes(c, M));
    int32_t* num_blocks = (int32_t*)((char*)workspace + schedule_bytes(c, M) - kAlign);
    int32_t* num_heavy = num_blocks + 1;
    const uint16_t* pgu = (const uint16_t*)W_packed;
    const uint16_t* pdn = pgu ? pgu + packed_gate_up_bytes(*c) / sizeof(uint16_t) : nullptr;
    hipError_t e = launch_block_schedule(*c, offsets, M, blocks, num_blocks, blocks_mix, num_heavy, s);
    if (e == hipSuccess)
        e = launch_gate_up(*c, M, (const uint16_t*)x_perm, c->d, nullptr, c->F, offsets, blocks, num_blocks, (const uint16_t*)W_gate,
                           (const uint16_t*)W_up, pgu, (uint16_t*)h, s);
    if (e == hipSuccess)
        e = launch_down(*c, M, (const uint16_t*)h, c->F, offsets, blocks, num_blocks, blocks_mix, num_heavy, (const uint16_t*)W_down, pdn,
                        (uint16_t*)y_perm, nullptr, s);
    return hip_status(e);
}

moe_status moe_combine(const moe_config* c, const void* y_perm, const int32_t* row_of, const float* topk_w,
                       void* y, void* stream) {
    const moe_status st = check_config(c);
    if (st != MOE_OK) return st;
    if (!y_perm || !row_of || !topk_w || !y) return MOE_ERR_NULL;
    if (misaligned(y_perm) || misaligned(y)) return MOE_ERR_ALIGN;
    if (c->T == 0) return MOE_OK;
    return hip_status(launch_combine(*c, (const uint16_t*)y_perm, row_of, topk_w, (uint16_t*)y,
                                     (hipStream_t)stream));
}

moe_status moe_forward_staged(const moe_config* c, const void* x, const void* W_r, const float* bias,
                              const void* W_gate, const void* W_up, const void* W_down, const void* W_packed,
                              void* y, void* workspace, size_t ws_bytes, void* stream, void* const* events,
                              int32_t n_events) {
    moe_workspace_layout l;
    const moe_status st = moe_forward_workspace_layout(c, &l);
    if (st != MOE_OK) return st;
    if (!x || !W_r || !y || !workspace) return MOE_ERR_NULL;
    if (!W_packed && (!W_gate || !W_up || !W_down)) return MOE_ERR_NULL;
    if (n_events < 0 || (n_events > 0 && events == nullptr)) return MOE_ERR_NULL;
    if (misaligned(x) || misaligned(W_r) || misaligned(W_gate) || misaligned(W_up) || misaligned(W_down) ||
        misaligned(y) || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0 ||
        (reinterpret_cast<uintptr_t>(W_packed) & (kAlign - 1)) != 0)
        return MOE_ERR_ALIGN;
    if (c->T == 0) return MOE_OK;   // nothing to do, so no workspace is needed either
    if (ws_bytes < l.total) return MOE_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    char* ws = (char*)workspace;
    const uint16_t* pgu = (const uint16_t*)W_packed;
    const uint16_t* pdn = pgu ? pgu + packed_gate_up_bytes(*c) / sizeof(uint16_t) : nullptr;
    int32_t* topk_idx = (int32_t*)(ws + l.topk_idx);
    float* topk_w = (float*)(ws + l.topk_w);
    int32_t* counts = (int32_t*)(ws + l.counts);
    int32_t* offsets = (int32_t*)(ws + l.offsets);
    int32_t* row_of = (int32_t*)(ws + l.row_of);
    int32_t* src_of = (int32_t*)(ws + l.src_of);
    uint16_t* h = (uint16_t*)(ws + l.h);
    uint16_t* y_perm = (uint16_t*)(ws + l.y_perm);
    void* route_ws = ws + l.scratch;
    int32_t* hist = (int32_t*)(ws + l.scratch + moe_route_workspace_size(c));
    const int M = moe_tile_m(c);
    int32_t* blocks = (int32_t*)((char*)hist + hist_bytes(c));
    int32_t* blocks_mix = (int32_t*)((char*)blocks + list_bytes(c, M));
    int32_t* num_blocks = (int32_t*)((char*)blocks + schedule_bytes(c, M) - kAlign);
    int32_t* num_heavy = num_blocks + 1;
    int32_t* arrive = (int32_t*)((char*)blocks + schedule_bytes(c, M));
    // Fold the weighted combine into the down projection when its kernel can (packed weights, the
    // per-block-regime kernels): the workgroup that writes the last of a token's k rows sums them.
    // On request only (MOE_FLAG_FUSE_COMBINE; a test knob can force it either way): with one
    // workgroup per CU nothing hides the latency of the epilogue's row reads, and from a few
    // hundred rows on that costs more than the combine launch it saves.
    const bool asked = knob(kKnobFuseCombine) >= 0 ? knob(kKnobFuseCombine) != 0 : (c->flags & MOE_FLAG_FUSE_COMBINE) != 0;
    const bool fuse = asked && down_fuses_combine(*c, M, pdn != nullptr);
    const CombineFusion fusion{src_of, row_of, topk_w, arrive, (uint16_t*)y};

    hipError_t e = hipSuccess;
    auto mark = [&](int i) {
        if (e == hipSuccess && i < n_events && events[i] != nullptr) e = hipEventRecord((hipEvent_t)events[i], s);
    };
    mark(0);
    if (e == hipSuccess)
        e = launch_route(*c, (const uint16_t*)x, (const uint16_t*)W_r, bias, topk_idx, topk_w, route_ws,
                         fuse ? arrive : nullptr, combine_groups(*c), s);
    mark(1);
    if (e == hipSuccess)
        e = launch_permute_index(*c, topk_idx, counts, offsets, row_of, src_of, hist, M, blocks, num_blocks, blocks_mix, num_heavy, s);
    mark(2);
    // The row gather of the permutation is folded into the gate+up tile loads (row r is read from
    // x[src_of[r] / k]); the permuted copy of x that moe_permute can write is not needed here.
    if (e == hipSuccess)
        e = launch_gate_up(*c, M, (const uint16_t*)x, c->d, src_of, c->F, offsets, blocks, num_blocks,
                           (const uint16_t*)W_gate, (const uint16_t*)W_up, pgu, h, s);
    mark(3);
    if (e == hipSuccess)
        e = launch_down(*c, M, h, c->F, offsets, blocks, num_blocks, blocks_mix, num_heavy, (const uint16_t*)W_down, pdn, y_perm,
                        fuse ? &fusion : nullptr, s);
    mark(4);
    if (e == hipSuccess && !fuse) e = launch_combine(*c, y_perm, row_of, topk_w, (uint16_t*)y, s);
    mark(5);
    return hip_status(e);
}

moe_status moe_forward(const moe_config* c, const void* x, const void* W_r, const float* bias, const void* W_gate,
                       const void* W_up, const void* W_down, const void* W_packed, void* y, void* workspace,
                       size_t ws_bytes, void* stream) {
    return moe_forward_staged(c, x, W_r, bias, W_gate, W_up, W_down, W_packed, y, workspace, ws_bytes, stream,
                              nullptr, 0);
}

}  // extern "C"
