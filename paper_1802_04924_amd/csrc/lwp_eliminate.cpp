// Single eliminations behind the C ABI: Eq. 2 (lwp_eliminate_node) and Eq. 3 (lwp_eliminate_edge).
#include "lwp_context.h"

using namespace lwp;

extern "C" {

// ---- Eq. 2 -------------------------------------------------------------------------------------
lwp_status lwp_eliminate_node(lwp_ctx* ctx, int32_t batch, int32_t Ci, int32_t Cj, int32_t Ck,
                              const int32_t* d_A, const int32_t* d_w, const int32_t* d_B,
                              int32_t* d_out, int32_t* d_argmin) {
    if (lwp_status s = check_ctx(ctx)) return s;
    if (batch < 1 || Ci < 1 || Cj < 1 || Ck < 1) return fail(ctx, LWP_E_INVAL, "sizes must be positive");
    if (Cj > kMaxConfigs) return fail(ctx, LWP_E_INVAL, "Cj exceeds 65536");
    if (!d_A || !d_w || !d_B || !d_out) return fail(ctx, LWP_E_INVAL, "null table pointer");
    if (((uintptr_t)d_A | (uintptr_t)d_w | (uintptr_t)d_B | (uintptr_t)d_out | (uintptr_t)d_argmin) & 3)
        return fail(ctx, LWP_E_INVAL, "table pointer not 4-byte aligned");
    const bool prefer_small = want_small_tiles(Ci, Cj, Ck, batch);
    if ((int64_t)((Ci + kTileSmall - 1) / kTileSmall) * ((Ck + kTileSmall - 1) / kTileSmall) * batch > 0x7fffffffLL)
        return fail(ctx, LWP_E_INVAL, "too many output tiles");

    // value ranges of A, w, B over the whole batch
    if (lwp_status s = ensure_workspace(ctx, 4096)) return s;
    if (lwp_status s = ensure_pinned(ctx, 4096)) return s;
    int32_t* d_stats = reinterpret_cast<int32_t*>(ctx->ws);
    LWP_HIP(ctx, launch_init_workspace(d_stats, 3, nullptr, nullptr, 0, ctx->stream));
    LWP_HIP(ctx, launch_ranges(d_A, 1, (int64_t)batch * Ci * Cj, d_stats, ctx->stream));
    LWP_HIP(ctx, launch_ranges(d_w, 1, (int64_t)batch * Cj, d_stats + 2, ctx->stream));
    LWP_HIP(ctx, launch_ranges(d_B, 1, (int64_t)batch * Cj * Ck, d_stats + 4, ctx->stream));
    int32_t* st = reinterpret_cast<int32_t*>(ctx->pin);
    LWP_HIP(ctx, hipMemcpyAsync(st, d_stats, 6 * sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
    LWP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    const Range rA{st[0], st[1]}, rw{st[2], st[3]}, rB{st[4], st[5]};
    if (!fits(rA.lo + rw.lo + rB.lo) || !fits(rA.hi + rw.hi + rB.hi) || !fits(rA.lo + rw.lo) || !fits(rA.hi + rw.hi))
        return fail(ctx, LWP_E_OVERFLOW, "A + w + B may leave int32");

    NodeArgs a{};
    a.descs = nullptr;
    a.base.A = d_A; a.base.w = d_w; a.base.B = d_B; a.base.out = d_out; a.base.arg = d_argmin;
    a.base.loA = (int32_t)rA.lo; a.base.hiA = (int32_t)rA.hi; a.base.loW = (int32_t)rw.lo; a.base.hiW = (int32_t)rw.hi;
    a.base.loB = (int32_t)rB.lo; a.base.hiB = (int32_t)rB.hi;
    const int64_t spread = keyed_spread(rA, rw, rB);
    // one more key bit on large tiles, worth it only if they still fill the chip; without an argmin
    // output the value-only variant runs, which has no range condition at all
    const bool value_only = (d_argmin == nullptr);
    const bool keyed = !value_only && (spread <= kKeyedMaxSpreadSmall ||
                       (spread <= kKeyedMaxSpreadLarge && (!prefer_small || large_tiles(Ci, Ck, batch) >= 512)));
    // keys re-based per row (64 x 64 tiles) where global offsets do not fit: only B's spread counts
    const bool keyed_row = !value_only && !keyed && keyed_row_spread(rB) <= kKeyedMaxSpreadSmall &&
                           keyed_row_pays(Ci, Cj, Ck, batch);
    const bool small = keyed_row || (prefer_small && (value_only || spread <= kKeyedMaxSpreadSmall || !keyed));
    const int tile = small ? kTileSmall : kTileLarge;
    const int64_t tilesM = (Ci + tile - 1) / tile, tilesN = (Ck + tile - 1) / tile;
    a.sA = (int64_t)Ci * Cj; a.sw = Cj; a.sB = (int64_t)Cj * Ck; a.sO = (int64_t)Ci * Ck;
    a.Ci = Ci; a.Cj = Cj; a.Ck = Ck; a.batch = batch;
    a.tilesM = (int32_t)tilesM; a.tilesN = (int32_t)tilesN;
    {
        ScopedTimer tm(ctx, 0, (int64_t)batch * Ci * Cj * Ck, keyed || keyed_row);
        const int kparts = choose_kparts(tilesM * tilesN * batch, Cj, small);
        if (kparts > 1) { if (lwp_status s = ensure_split_buffers(ctx)) return s; }
        set_split(ctx, a, kparts);
        LWP_HIP(ctx, launch_minplus(a, value_only ? kModeValue : (keyed ? kModeKeyed : (keyed_row ? kModeKeyedRow : kModePlain)), small, ctx->stream));
    }
    return LWP_OK;
}

// ---- Eq. 3 -------------------------------------------------------------------------------------
lwp_status lwp_eliminate_edge(lwp_ctx* ctx, int32_t batch, int32_t Ci, int32_t Cj,
                              const int32_t* d_e1, const int32_t* d_e2, int32_t* d_out) {
    if (lwp_status s = check_ctx(ctx)) return s;
    if (batch < 1 || Ci < 1 || Cj < 1) return fail(ctx, LWP_E_INVAL, "sizes must be positive");
    if (!d_e1 || !d_e2 || !d_out) return fail(ctx, LWP_E_INVAL, "null table pointer");
    if (((uintptr_t)d_e1 | (uintptr_t)d_e2 | (uintptr_t)d_out) & 3)
        return fail(ctx, LWP_E_INVAL, "table pointer not 4-byte aligned");
    const int64_t cells = (int64_t)batch * Ci * Cj;
    ScopedTimer tm(ctx, 1, cells, false);
    LWP_HIP(ctx, launch_edge_sum_pair(d_e1, d_e2, d_out, cells, ctx->stream));
    return LWP_OK;
}

}  // extern "C"
