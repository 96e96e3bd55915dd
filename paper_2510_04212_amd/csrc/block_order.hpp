// Order in which the work-groups of a small causal grid take their blocks.
//
// Under the causal mask the blocks of one head differ in work by up to nblk : 1.  When the whole
// grid (or most of it) is resident at once, how long the kernel runs is decided by the compute
// unit whose work-groups add up to the most work, and the hardware places work-groups by a fixed
// rule: the grid goes round-robin over the 8 XCDs, and inside an XCD the s-th work-group goes to
// compute unit s mod 32 for as long as slots are free (observed by recording each work-group's
// hardware id: with three work-groups per unit resident, s, s + 32 and s + 64 share a unit).
// A fixed heavy-to-light order per head then stacks blocks of the same weight class on the same
// unit.  This table gives the s-th work-group of an XCD the work item pos[s] of that XCD's share
// instead, chosen so that the resident work-groups of every unit carry nearly the same total
// (longest-processing-time greedy over the units); items beyond what is resident at once follow
// heaviest first and are picked up by whichever unit frees a slot.
//
// Plain C++ (no HIP): the struct is a kernel argument, the fill routine runs on the host.
#pragma once
#include <algorithm>

constexpr int kCUsPerXCD = 32;
constexpr int kMaxOrder = 255;

struct BlockOrder {
  unsigned short n;                 // entries in use; 0 = no table, work-groups keep their own order
  unsigned short pos[kMaxOrder];
};

// per: work items of one XCD (grid / 8), item j being block (j % nblk) of some head, in the
// kernels' heavy-first numbering: its work is proportional to nblk - j % nblk key (or query)
// tiles plus a fixed start-up share.  resident: work-groups of this kernel a compute unit holds
// at once.  Returns false (and n = 0) when the table does not apply.
inline bool fill_block_order(BlockOrder& ord, int per, int nblk, int resident) {
  ord.n = 0;
  if (per <= 0 || per > kMaxOrder || nblk <= 0 || per % nblk != 0 || resident <= 0) return false;
  auto weight = [&](int j) { return 2 * (nblk - j % nblk) + 1; };
  // the items by falling weight (heads in their own order within a weight class); no heap use,
  // the routine runs inside kernel launches
  unsigned short items[kMaxOrder];
  for (int idx = 0, n = 0; idx < nblk; ++idx)
    for (int first = 0; first < per; first += nblk) items[n++] = (unsigned short)(first + idx);
  const int slots = std::min(per, kCUsPerXCD * resident);       // positions that are placed at launch
  int cap[kCUsPerXCD], cnt[kCUsPerXCD], load[kCUsPerXCD];
  for (int c = 0; c < kCUsPerXCD; ++c) {
    cap[c] = slots / kCUsPerXCD + (c < slots % kCUsPerXCD ? 1 : 0);
    cnt[c] = 0;
    load[c] = 0;
  }
  for (int i = 0; i < slots; ++i) {                             // heaviest first, onto the least loaded unit
    int best = -1;
    for (int c = 0; c < kCUsPerXCD; ++c)
      if (cnt[c] < cap[c] && (best < 0 || load[c] < load[best])) best = c;
    ord.pos[cnt[best] * kCUsPerXCD + best] = (unsigned short)items[i];
    ++cnt[best];
    load[best] += weight(items[i]);
  }
  for (int i = slots; i < per; ++i) ord.pos[i] = (unsigned short)items[i];
  ord.n = (unsigned short)per;
  return true;
}
