// Internal declarations shared by the translation units of libwlb (not installed).
#pragma once
#include <cstdarg>
#include <cstddef>
#include <cstdint>

#include "wlb.h"

namespace wlb {

// Records the text returned by wlb_last_error() on this thread and passes `st` through.
wlb_status fail(wlb_status st, const char* fmt, ...);

constexpr int kGroupRows = 64;    // rows per schedule group (granularity of hull / full-range data)
constexpr int kFwdTileRows = 128; // query rows per forward / dQ work item
constexpr int kBwdKeyTile = 128;  // keys per dK/dV work item

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr int kLists = 8;         // XCDs: workgroup b runs on XCD b % 8
// Short-hull path of the forward and dQ kernels: a block of 32 rows whose visible keys, counted from
// the 32-key boundary at or below the first, span at most kShortHullKeys keys is worked on by one
// workgroup that holds those K/V rows in LDS for all query heads of the KV head.  A query tile
// takes this path when each of its four blocks qualifies.
constexpr int kShortBlockRows = 32;
constexpr int kShortHullKeys = 96;
#ifndef WLB_DKV_SPLIT
#define WLB_DKV_SPLIT 6
#endif
constexpr int kDkvSplit = WLB_DKV_SPLIT;      // a dK/dV item is at most 1/kDkvSplit of the mean load of a compute unit
#ifndef WLB_DKV_MIN_ITEM_STAGES
#define WLB_DKV_MIN_ITEM_STAGES 32
#endif
constexpr int kDkvMinItemStages = WLB_DKV_MIN_ITEM_STAGES;   // items this short are never split further
constexpr int kMergeSplit = 4;     // workgroups per cut query tile and head in the merge kernels (rows split evenly)

// compute units of the GPU (256 when none is present: layout queries on the host)
int compute_units();
// Forward and dQ run as a fixed set of workgroups, two per compute unit, in gangs of the
// G = hq / hkv query heads that share a KV head (a gang's workgroups sit on one XCD and walk the
// same K/V tiles side by side).  Number of gangs:
inline int row_gangs(int hq, int hkv, int cus) {
    const int per_xcd = (2 * cus / kLists) / (hq / hkv);
    return kLists * (per_xcd > 0 ? per_xcd : 1);
}
// fixed cost of a query tile (loading Q, the first copies, the output) in units of one key tile's work
constexpr int kRowItemOverhead = 6;
// Default relative work share (percent) of a gang of the first half of a launch; a gang of the second half
// gets the rest.  Set from the gangs' recorded end times (wlb_plan_layout: off_gang_clock): with these shares
// the two halves end together on average.  What remains is a spread between the XCDs of a GPU (one XCD's
// gangs end several percent later than another's, the same ones in every launch), which differs from GPU to
// GPU: wlb_attn_set_gang_weights takes weights measured on the GPU at hand.
constexpr int kRowShareFirstFwd = 57, kRowShareFirstDq = 57;
// the weights in force for kernel 0 (forward) / 1 (dQ): [half of the launch][XCD]
void gang_weights(int kernel, int out[2][8]);
// Which of the two forward / dQ schedules a launch uses: gangs with fixed shares when there are fewer
// than kRowGangMaxItemsPerSlot (query tile, head) items per workgroup slot and an estimated
// kRowGangMinUnitsPerSlot key tiles of work per slot, else one workgroup per item.  The
// WLB_ATTN_SCHEDULE_* flags override.
constexpr int kRowGangMaxItemsPerSlot = 3;
constexpr int kRowGangMinUnitsPerSlot = 64;
bool use_row_gangs(const wlb_attn_desc& d, const wlb_plan_layout& L);
// whether this launch sends short-hull query tiles to the short-hull kernels (only in the
// one-workgroup-per-item schedule; WLB_ATTN_NO_SHORT_PATH switches it off)
bool use_short_path(const wlb_attn_desc& d, const wlb_plan_layout& L);
// floats of one partial result of a query tile and head: 128 x D accumulator, then 128 row sums and
// 128 reference exponents
inline size_t row_partial_floats(int head_dim) { return (size_t)kFwdTileRows * head_dim + 2 * kFwdTileRows; }
// bytes of the partial results of the query tiles that are cut at a gang boundary: two per gang and member
size_t row_partial_bytes(const wlb_attn_desc& d, const wlb_plan_layout& L);
// bytes of the dK/dV partial results that follow delta / lse2 in the backward workspace
size_t dkv_partial_bytes(const wlb_attn_desc& d, const wlb_plan_layout& L);

// Validates desc; on success fills the plan layout.
wlb_status check_desc(const wlb_attn_desc* d);
void plan_layout(const wlb_attn_desc& d, wlb_plan_layout* L);

// Device-side launchers (defined in the .hip files); all asynchronous on `stream`.
wlb_status launch_plan(const wlb_attn_desc& d, const wlb_plan_layout& L, const int32_t* q_idx,
                       const int32_t* cu_seqlens_k, char* ws, void* stream);
wlb_status launch_fwd(const wlb_attn_desc& d, const wlb_plan_layout& L, const void* q, const void* k,
                      const void* v, void* o, float* lse, char* ws, size_t off_row_partial, void* stream);
wlb_status launch_bwd(const wlb_attn_desc& d, const wlb_plan_layout& L, const void* q, const void* k,
                      const void* v, const void* o, const float* lse, const void* d_o, void* dq,
                      void* dk, void* dv, char* ws, size_t off_delta, void* stream);

}  // namespace wlb
