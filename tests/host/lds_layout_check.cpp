// Host check of the LDS layout the matmul kernels use (csrc/lds_layout.h): emulates, with the very index
// functions the kernels call, the direct loads of one operand slab and every fragment read of every wavefront,
// for each tile size and both memory orders, and checks that
//   * every global offset addresses the element it should and every LDS byte is filled exactly once,
//   * every fragment read stays inside the slab and returns the rows and k the MFMA expects,
//   * reads are free of LDS bank conflicts (64 banks of 4 bytes).
// The transposing read of gfx950 (ds_read_b64_tr_b16) is modelled as measured on the hardware: within a group
// of sixteen lanes, lane i receives as element m (m = 0..3) element i % 4 of what lane 4 m + i / 4 addressed.
#include <cstdio>
#include <cstdlib>
#include <map>
#include <utility>
#include <vector>

#include "lds_layout.h"

using dash::layout::F32;
using dash::layout::Half;

static int failures = 0;
#define CHECK(cond, ...) do { if (!(cond)) { ++failures; std::printf("FAIL %s:%d: ", __FILE__, __LINE__); std::printf(__VA_ARGS__); std::printf("\n"); if (failures > 20) std::exit(1); } } while (0)

typedef std::pair<int, int> Elem;      // (row of the tile, k of the slab)

template <int TILE, int HBK, int NW, int WT>
static void check_half(bool kc) {
    typedef Half<TILE, HBK, NW> L;
    const int ld = 1024, row0 = 256;
    const int WC = TILE / WT, MT = WT / 32;
    std::map<int, Elem> lds;            // LDS byte offset of a 16-bit element -> what it holds
    for (int wave = 0; wave < NW; ++wave)
        for (int lane = 0; lane < 64; ++lane)
            for (int u = 0; u < L::NV; ++u) {
                const unsigned off = L::load_offset(kc, ld, row0, wave, lane, u);
                CHECK(off % 16 == 0, "unaligned source cell");
                const int dst = L::chunk(wave, u) * 1024 + lane * 16;
                CHECK(dst + 16 <= L::SLAB, "chunk outside the slab");
                for (int e = 0; e < 8; ++e) {
                    const int g = (int)(off / 2) + e;          // element index inside the block
                    Elem el = kc ? Elem(g / ld - row0, g % ld) : Elem(g % ld - row0, g / ld);
                    CHECK(el.first >= 0 && el.first < TILE && el.second >= 0 && el.second < HBK,
                          "TILE %d %s: lane fetches (%d, %d)", TILE, kc ? "KC" : "KR", el.first, el.second);
                    CHECK(!lds.count(dst + 2 * e), "LDS byte written twice");
                    lds[dst + 2 * e] = el;
                }
            }
    CHECK((int)lds.size() == TILE * HBK, "slab not covered: %zu of %d", lds.size(), TILE * HBK);
    int worst = 0;
    for (int wave = 0; wave < NW; ++wave)
        for (int side = 0; side < 2; ++side) {              // as row operand (wm) and as column operand (wn)
            const int r0 = (side == 0 ? wave / WC : wave % WC) * WT;
            for (int i = 0; i < MT; ++i)
                for (int st = 0; st < L::STEPS; ++st) {
                    if (kc) {
                        for (int g0 = 0; g0 < 64; g0 += 16) {          // a 16-byte read is served 16 lanes at a time
                            std::map<int, int> groups;
                            for (int lane = g0; lane < g0 + 16; ++lane) {
                                const int a = L::frag_kc(r0, lane, st) + i * L::KC_SUB;
                                CHECK(a >= 0 && a + 16 <= L::SLAB && a % 16 == 0, "KC read outside the slab");
                                for (int e = 0; e < 8; ++e) {
                                    const Elem want(r0 + 32 * i + (lane & 31), 16 * st + 8 * (lane >> 5) + e);
                                    CHECK(lds[a + 2 * e] == want, "TILE %d KC lane %d step %d: wrong element", TILE, lane, st);
                                }
                                worst = std::max(worst, ++groups[(a / 16) % 16]);
                            }
                        }
                    } else {
                        for (int h = 0; h < 2; ++h) {
                            std::vector<std::vector<Elem>> loaded(64);
                            for (int g0 = 0; g0 < 64; g0 += 32) {      // an 8-byte read is served 32 lanes at a time
                                std::map<int, int> banks;
                                for (int lane = g0; lane < g0 + 32; ++lane) {
                                    const int a = L::frag_kr(r0, i, lane) + st * L::KR_STEP + h * L::KR_HALF;
                                    CHECK(a >= 0 && a + 8 <= L::SLAB && a % 8 == 0, "KR read outside the slab");
                                    for (int e = 0; e < 4; ++e) loaded[lane].push_back(lds[a + 2 * e]);
                                    for (int d = 0; d < 2; ++d) worst = std::max(worst, ++banks[(a / 4 + d) % 64]);
                                }
                            }
                            for (int lane = 0; lane < 64; ++lane) {
                                const int blk = lane & ~15, ii = lane & 15;
                                for (int m = 0; m < 4; ++m) {
                                    const Elem got = loaded[blk + 4 * m + ii / 4][ii % 4];
                                    const Elem want(r0 + 32 * i + (lane & 31), 16 * st + 8 * (lane >> 5) + 4 * h + m);
                                    CHECK(got == want, "TILE %d KR lane %d step %d half %d: got (%d, %d) want (%d, %d)", TILE, lane,
                                          st, h, got.first, got.second, want.first, want.second);
                                }
                            }
                        }
                    }
                }
        }
    CHECK(worst == 1, "TILE %d %s: bank multiplicity %d", TILE, kc ? "KC" : "KR", worst);
    std::printf("16-bit TILE %3d HBK %d %s: placement, fragments and banks ok\n", TILE, HBK, kc ? "KC" : "KR");
}

template <int TILE, int BK, int NW, int WT>
static void check_f32(bool kc) {
    typedef F32<TILE, BK, NW> L;
    const int ld = 1024, row0 = 384;
    const int WC = TILE / WT, MT = WT / 32;
    std::map<int, Elem> lds;            // LDS float offset -> what it holds
    for (int wave = 0; wave < NW; ++wave)
        for (int lane = 0; lane < 64; ++lane)
            for (int u = 0; u < L::NV; ++u) {
                const unsigned off = L::load_offset(kc, ld, row0, wave, lane, u);
                CHECK(off % 16 == 0, "unaligned source cell");
                const int dst = L::chunk(wave, u) * 256 + lane * 4;
                CHECK(dst + 4 <= L::SLAB, "chunk outside the slab");
                for (int e = 0; e < 4; ++e) {
                    const int g = (int)(off / 4) + e;
                    Elem el = kc ? Elem(g / ld - row0, g % ld) : Elem(g % ld - row0, g / ld);
                    CHECK(el.first >= 0 && el.first < TILE && el.second >= 0 && el.second < BK,
                          "fp32 TILE %d %s: lane fetches (%d, %d)", TILE, kc ? "KC" : "RC", el.first, el.second);
                    CHECK(!lds.count(dst + e), "LDS float written twice");
                    lds[dst + e] = el;
                }
            }
    CHECK((int)lds.size() == L::SLAB, "slab not covered");
    int worst = 0;
    for (int wave = 0; wave < NW; ++wave)
        for (int side = 0; side < 2; ++side) {
            const int r0 = (side == 0 ? wave / WC : wave % WC) * WT;
            for (int i = 0; i < MT; ++i)
                for (int c = 0; c < BK / 8; ++c) {
                    if (kc) {
                        for (int g0 = 0; g0 < 64; g0 += 16) {
                            std::map<int, int> groups;
                            for (int lane = g0; lane < g0 + 16; ++lane) {
                                const int a = L::frag_kc(r0, lane, c) + i * L::KC_SUB;
                                CHECK(a >= 0 && a + 4 <= L::SLAB && a % 4 == 0, "KC read outside the slab");
                                for (int s = 0; s < 4; ++s)
                                    CHECK(lds[a + s] == Elem(r0 + 32 * i + (lane & 31), 8 * c + 4 * (lane >> 5) + s),
                                          "fp32 TILE %d KC lane %d chunk %d: wrong element", TILE, lane, c);
                                worst = std::max(worst, ++groups[(a / 4) % 16]);
                            }
                        }
                    } else {
                        for (int s = 0; s < 4; ++s) {
                            std::map<int, int> banks;
                            for (int lane = 0; lane < 64; ++lane) {
                                const int a = L::frag_rc(r0, i, lane) + (8 * c + s) * TILE;
                                CHECK(a >= 0 && a < L::SLAB, "RC read outside the slab");
                                CHECK(lds[a] == Elem(r0 + 32 * i + (lane & 31), 8 * c + 4 * (lane >> 5) + s),
                                      "fp32 TILE %d RC lane %d chunk %d step %d: wrong element", TILE, lane, c, s);
                                worst = std::max(worst, ++banks[a % 64]);
                            }
                        }
                    }
                }
        }
    CHECK(worst == 1, "fp32 TILE %d %s: bank multiplicity %d", TILE, kc ? "KC" : "RC", worst);
    std::printf("fp32   TILE %3d BK %d %s: placement, fragments and banks ok\n", TILE, BK, kc ? "KC" : "RC");
}

int main() {
    for (int kc = 0; kc < 2; ++kc) {
        check_half<64, 64, 4, 32>(kc);          // the three instantiations of the 16-bit kernel
        check_half<128, 64, 4, 64>(kc);
        check_half<256, 64, 16, 64>(kc);
        check_half<256, 32, 16, 64>(kc);        // slabs of 32 (ring of 3 to 5 stages)
        check_f32<64, 16, 4, 32>(kc);           // the fp32 kernel
        check_f32<128, 16, 4, 64>(kc);
        check_f32<128, 32, 4, 64>(kc);
        check_f32<256, 16, 16, 64>(kc);
    }
    if (failures) { std::printf("%d failures\n", failures); return 1; }
    std::printf("all layouts ok\n");
    return 0;
}
