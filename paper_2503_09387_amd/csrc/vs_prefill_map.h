// Where the workgroups of a bf16 prefill launch go when the key splits are merged inside the
// kernel; the dense layers' split-K launches place their workgroups the same way (unit = block of
// output features, split = share of the input features).  Shared by the kernels, the launchers
// and a host-side test (plain C++, no HIP types).
//
// The merge goes through the L2 cache that the compute units of one XCD share, so all splits
// of a unit = (KV head, frame, row tile) must run on one XCD.  The hardware deals workgroup ids
// to the XCDs in turn (id mod number of XCDs; read off the device once, and checked again by
// every workgroup of every launch).  Unit u therefore takes the ids of one residue x:
//     x = u / units_per_xcd,  j = u % units_per_xcd,  id = x + ((j * nsplit + split) << xcd_shift)
// with units_per_xcd = ceil(units / 2^xcd_shift); consecutive units (the same KV head, whose K/V
// that L2 then holds once) share an XCD.  Ids whose unit does not exist are spare and return.
#pragma once

#ifdef __HIPCC__
#define VS_HD __host__ __device__ __forceinline__
#else
#define VS_HD inline
#endif

namespace vs {

// floor(x / d) for 0 <= x < 2^22 and d >= 1, given inv_d = 1.0f / d: the float product is within
// one of the quotient, two corrections make it exact.  (A 32-bit integer division costs some
// twenty instructions on the device, and the prologue of the prefill kernel is on its critical
// path.)
VS_HD int div_small(int x, int d, float inv_d) {
    int qd = (int)((float)x * inv_d);
    if (qd * d > x) --qd;
    if ((qd + 1) * d <= x) ++qd;
    return qd;
}

struct PrefillSlot {
    int unit;   // -1: a spare id
    int split;
    int xcd;    // residue of the id: which XCD of the dealing order it lands on
};

VS_HD int prefill_units_per_xcd(int units, int xcd_shift) { return (units + (1 << xcd_shift) - 1) >> xcd_shift; }

VS_HD unsigned prefill_grid_ids(int units, int nsplit, int xcd_shift) {
    return (unsigned)(prefill_units_per_xcd(units, xcd_shift) * nsplit) << xcd_shift;
}

VS_HD PrefillSlot prefill_slot_of_id(unsigned id, int units, int units_per_xcd, int nsplit, float inv_nsplit,
                                     int xcd_shift) {
    PrefillSlot s;
    s.xcd = (int)(id & ((1u << xcd_shift) - 1u));
    const int slot = (int)(id >> xcd_shift);
    const int j = div_small(slot, nsplit, inv_nsplit);
    s.split = slot - j * nsplit;
    s.unit = s.xcd * units_per_xcd + j;
    if (j >= units_per_xcd || s.unit >= units) s.unit = -1;
    return s;
}

}  // namespace vs
