// ss_embbag_forward_grouped: the pooled lookup and the grouping half of the
// backward pass in one launch.
//
// Grouping a table's lookups by row needs only the indices, which the forward
// pass reads anyway, and it is bound by latency and LDS/VALU work on a few
// hundred workgroups while the gather is bound by HBM.  Launched one after the
// other they cost their sum; as two roles of one grid the grouping workgroups
// (lowest block ids, dispatched first) run in the shadow of the gather.  The
// grouping role sorts 31-bit words (row bits above the class bits + sample
// number), which keeps its LDS small enough for two 1024-thread workgroups per
// CU, so the gather role keeps its occupancy.
#include "forward_body.h"
#include "group_body.h"
#include "ss_common.h"

namespace ss {

template <int G, int ITEMS>
__global__ __launch_bounds__(1024) void forward_group_kernel(
    const float *const *__restrict__ weights, const int32_t *__restrict__ idx,
    int Bcap, const int32_t *__restrict__ n_valid, float *__restrict__ out, int D4,
    int tiles_per_table, const uint32_t *const *__restrict__ bits,
    int key_bits, int class_bits, int val_bits, uint2 *__restrict__ out_ent, int NP,
    int group_blocks, bool interleave)
{
    // Roles are interleaved (one grouping workgroup, two gather workgroups, ...)
    // while both last, so that every CU starts with a mix of the two.
    const int b = blockIdx.x;
    int gb = -1, fb;
    if (interleave && b < 3 * group_blocks) {
        if (b % 3 == 0) gb = b / 3;
        fb = b - b / 3 - 1;
    } else if (!interleave && b < group_blocks) {
        gb = b;
        fb = 0;
    } else {
        fb = b - group_blocks;
    }
    if (gb >= 0) {
        const int classes = 1 << class_bits;
        class_sort_body<ITEMS, true>(gb % classes, gb / classes, idx, Bcap, 1, n_valid,
                                     bits, key_bits, class_bits, val_bits, out_ent, NP);
    } else {
        forward_onehot_body<G, 1024>(fb, weights, idx, Bcap, n_valid, out, D4,
                                     tiles_per_table);
    }
}

bool can_fuse_forward_group(const ss_tables *tb, int Bcap, int L)
{
    if (L != 1) return false;
    const int NP = (int)align_up((size_t)Bcap, 2048);
    if (NP > 16384) return false;
    int key_bits = 1;
    while (key_bits < 31 && (1LL << key_bits) < tb->rows) ++key_bits;
    return plan_class_sort(NP, Bcap, key_bits).packed;
}

int32_t launch_forward_group(const ss_tables *tb, const int32_t *idx, int Bcap,
                             const int32_t *n_valid, float *out, uint2 *ent, int NP,
                             hipStream_t s)
{
    const int T = tb->num_tables, D4 = tb->dim / 4;
    int key_bits = 1;
    while (key_bits < 31 && (1LL << key_bits) < tb->rows) ++key_bits;
    const ClassSortPlan cp = plan_class_sort(NP, Bcap, key_bits);
    const int g = lanes_per_row(tb->dim);
    const int bags = (1024 / g) * kOneHotBags;
    const int tiles = (Bcap + bags - 1) / bags;
    const int group_blocks = T << cp.class_bits;
    const int64_t blocks = (int64_t)tiles * T + group_blocks;
    if (blocks > 0x7fffffffLL)
        return fail(SS_ERR_UNSUPPORTED, "ss_embbag_forward_grouped: grid too large");
    ProfScope prof("forward_group_kernel", s);
#define SS_FG(I)                                                                    \
    SS_DISPATCH_G(g, launch(forward_group_kernel<G, I>, dim3((unsigned)blocks),     \
                            dim3(1024), s, tb->weights, idx, Bcap, n_valid, out, D4, \
                            tiles, tb->stale_bits, key_bits, cp.class_bits,   \
                            cp.val_bits, ent, NP, group_blocks,                     \
                            (int64_t)tiles * T >= 2 * (int64_t)group_blocks))
    if (cp.items == 2) { SS_FG(2); }
    else if (cp.items == 4) { SS_FG(4); }
    else if (cp.items == 8) { SS_FG(8); }
    else { SS_FG(16); }
#undef SS_FG
    return check_launch("ss_embbag_forward_grouped");
}

}  // namespace ss
