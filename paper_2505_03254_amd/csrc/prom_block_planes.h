// The block kernel that keeps the expanded tensor in LDS as 16-channel planes: arguments, planning
// and launch (prom_block_planes.hip), used by prom_block_ex (prom_block.hip).
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace prom {

struct PlanesArgs {
    const int8_t *x;
    int8_t *y;
    const uint32_t *we;  // packed expand weights [chid][cin]
    const int8_t *wd;    // depthwise weights [3][3][chid]
    const uint32_t *wp;  // packed project weights [cout][chid]
    const int32_t *be, *me, *se;  // expand bias / mult / shift [chid]
    const int32_t *bd, *md, *sd;  // depthwise [chid]
    const int32_t *bp, *mp, *sp;  // project [cout]
    const int32_t *ne, *nd, *np;  // PReLU negative-side multipliers of the three layers, or nullptr
    int N, H, W, Ho, Wo, cin, chid, cout, stride;
    int R, bands, RI;  // output rows per band, bands per image, plane rows = (R-1)*stride + 3
    int add_res;
    int lo_e, hi_e, lo_d, hi_d, lo_p, hi_p;
    int NW;             // wavefronts per workgroup: 8, 12 or 16
    int NP, COT;        // 16-channel planes of the hidden tensor, 16-channel tiles of the output
    int KWe, KWp, KS3;  // packed words per expand / project weight row, k steps of the projection
    int cinp;           // bytes between pixels of the band's input in LDS
    int G1, G2;         // wavefront units per plane in phases 1 and 2 (1: a plane has one owner)
    int G3, TPG3;       // phase 3: pixel-tile groups per output tile, pixel tiles per group (1, 2, 4 or 8)
    int slot1, slot2;   // bytes between expansion planes / between depthwise-output planes
    int S3;             // words between rows of the projection's packed codes in LDS
    int off_o1, off_o2, off_pp, off_w3, off_wd, off_t1, off_t2;  // LDS byte offsets
};

// Band height, unit split and LDS layout for the shape in `a`; false if the kernel does not take it.
bool plan_planes(PlanesArgs &a, size_t &lds, int &grid, int &kse);
// Launch; PROM_OK or PROM_EHIP.
int launch_planes(const PlanesArgs &a, size_t lds, int grid, int kse, void *stream);

}  // namespace prom
