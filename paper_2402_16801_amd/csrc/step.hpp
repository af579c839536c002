// One Craftax-Classic step of one environment, executed by the G lanes that own it.
//
// What the paper fixes: 17 actions that are always legal and fall back to a no-op when their
// prerequisites are missing (section "RL Environment Interface"), 22 achievements worth +1
// the first time and +-0.1 per health point (same section), fixed-capacity creature and plant
// tables whose empty slots are masked (appendix "Differences between Craftax-Classic and
// Crafter"), creature health and damage (appendix "Creatures").  The remaining rules
// ("mimic Crafter") are this library's own frozen reading.
//
// Random draws have fixed slots: Philox block k (k = 0..11) of the step =
// (move draw of mob k, decision draw of mob k, eaten draw of plant k, misc[k]);
// misc[3j..3j+2] = (x, y, p) of the spawn attempt of type j; misc[9] = sapling draw.
//
// Memory round trips of a step: record -> 9x11 map window around the player (kept in LDS,
// patched with this step's edits, and reused for the observation) -> one terrain byte per
// moving mob and per spawn candidate.
#pragma once

#include "common.hpp"

namespace cx {

enum Intent : int { K_NONE = 0, K_MOVE = 1, K_MOVE_PATH = 2, K_ATTACK = 3, K_SHOOT = 4, K_FLY = 5 };

struct StepOut { bool done; float reward; int mvx, mvy; };

// Loads the 9x11 window centred on (px, py) into LDS; cells outside the map read as BK_OOB.
template <int G>
__device__ inline void load_window(int l, int px, int py, const uint8_t* __restrict__ map, uint8_t* win)
{
#pragma unroll
    for (int it_i = 0; it_i < ((WIN_CELLS) + G - 1) / G; ++it_i) {
        const int i = l + it_i * G;
        if (i >= (WIN_CELLS)) break;
        const int r = i / WIN_COLS, c = i - r * WIN_COLS;
        const int x = px - WIN_COLS / 2 + c, y = py - WIN_ROWS / 2 + r;
        win[i] = in_map(x, y) ? map[y * MAPW + x] : (uint8_t)BK_OOB;
    }
}

// e: the environment's LDS area (record already loaded).  Returns with the record in LDS
// updated (unless the episode ended) and the window patched with this step's map edits;
// (mvx, mvy) is how far the player moved, i.e. where the view sits inside the window.
template <int G>
__device__ inline StepOut step_env(int l, uint32_t env, uint32_t* e, uint8_t* __restrict__ map,
                                   const Luts* __restrict__ luts, int action, const Params& p)
{
    using Gr = Grp<G>;
    constexpr int NSM = Gr::NS_MOB, NSP = Gr::NS_PLANT;
    uint32_t* rec = e + LDS_REC;
    uint8_t* win = reinterpret_cast<uint8_t*>(e + LDS_WIN);

    // ---- unpack -----------------------------------------------------------------------------
    const uint32_t w_pos = rec[RW_POS], w_inv = rec[RW_INV], w_vit = rec[RW_VIT], w_cnt = rec[RW_CNT];
    const int px0 = w_pos & 0xFF, py0 = (w_pos >> 8) & 0xFF;
    int px = px0, py = py0, dir = (w_pos >> 16) & 0xFF, sleeping = (w_pos >> 24) & 0xFF;
    int inv[12], vit[4], cnt[4];
#pragma unroll
    for (int i = 0; i < 6; ++i) { inv[i] = (w_inv >> (4 * i)) & 15; inv[6 + i] = (w_inv >> (24 + i)) & 1; }
#pragma unroll
    for (int i = 0; i < 4; ++i) { vit[i] = (w_vit >> (4 * i)) & 15; cnt[i] = (int)(int8_t)(w_cnt >> (8 * i)); }
    uint32_t phase = w_vit >> 16;
    uint32_t ach = rec[RW_ACH];
    const uint32_t t = rec[RW_T], episode = rec[RW_EPISODE], seed_lo = rec[RW_SEED_LO], seed_hi = rec[RW_SEED_HI];
    Mob m[NSM];
    U4 dr[NSM];
#pragma unroll
    for (int s = 0; s < NSM; ++s) {
        const int k = l + s * G;
        m[s] = unpack_mob(k < NMOB ? rec[RW_MOB + k] : 0u);
        dr[s] = philox4x32_10(env, t, episode, (DOM_STEP << 16) | (uint32_t)k, seed_lo, seed_hi);
    }
    Plant q[NSP];
    int q_block[NSP];
#pragma unroll
    for (int s = 0; s < NSP; ++s) {
        const int k = l + s * G;
        q[s] = unpack_plant(k < NPLANT ? rec[RW_PLANT + k] : 0u);
        q_block[s] = q[s].alive ? (int)map[q[s].y * MAPW + q[s].x] : (int)BK_INVALID;
    }
    const int health0 = vit[0];
    const uint32_t ach0 = ach;

    load_window<G>(l, px0, py0, map, win);
    const uint32_t sapling_draw = (uint32_t)Gr::shfl((int)dr[9 / G].w[3], 9 % G);

    int a = ((unsigned)action < (unsigned)AC_COUNT) ? action : (int)AC_NOOP;
    if (sleeping) a = AC_NOOP;
    group_sync();   // the window is in LDS

    // ---- phase 1: the player's action ----------------------------------------------------------
    bool l_table = false, l_furnace = false;
#pragma unroll
    for (int it_j = 0; it_j < ((9) + G - 1) / G; ++it_j) {
        const int j = l + it_j * G;
        if (j >= (9)) break;
        const int b = win[(3 + j / 3) * WIN_COLS + 4 + j % 3];
        l_table = l_table || b == BK_TABLE;
        l_furnace = l_furnace || b == BK_FURNACE;
    }
    const bool near_table = Gr::ballot(l_table) != 0, near_furnace = Gr::ballot(l_furnace) != 0;

    if (a >= AC_LEFT && a <= AC_DOWN) dir = a;
    const int ddx = dir_dx(dir), ddy = dir_dy(dir);
    const int fx = px + ddx, fy = py + ddy;
    const bool f_in = in_map(fx, fy);
    const int f_win = (WIN_ROWS / 2 + ddy) * WIN_COLS + WIN_COLS / 2 + ddx;
    const int fb = win[f_win];
    // which mob (if any) stands on the facing cell: owner lane and sub-slot
    int my_hit = -1;
#pragma unroll
    for (int s = 0; s < NSM; ++s)
        if (m[s].alive && m[s].x == fx && m[s].y == fy) my_hit = s | (m[s].hp << 4);
    const uint32_t hit_lanes = Gr::ballot(my_hit >= 0);
    const int hit_lane = hit_lanes ? (__ffs((int)hit_lanes) - 1) : -1;
    const int hit_info = Gr::shfl(my_hit, hit_lane < 0 ? 0 : hit_lane);
    const int hit = hit_lane < 0 ? -1 : hit_lane + G * (hit_info & 15);   // mob slot index
    const int hit_hp = hit_info >> 4;
    uint32_t plant_mask = 0;
#pragma unroll
    for (int s = 0; s < NSP; ++s) plant_mask |= Gr::ballot(q[s].alive != 0) << (s * G);

    int modval = -1;                 // new block of the facing cell, if the action edits it
    bool ate_ripe = false;
    int new_plant_slot = -1;

    if (a >= AC_LEFT && a <= AC_DOWN) {
        if (f_in && hit < 0) {
            if (walkable_ground(fb)) { px = fx; py = fy; }
            else if (fb == BK_LAVA) { px = fx; py = fy; vit[0] = 0; }
        }
    } else if (a == AC_DO) {
        if (f_in) {
            if (hit >= 0) {
                const int type = (hit * 11) >> 5;
                if (type != MT_ARROW) {
                    const int dmg = inv[IV_IRON_SWORD] ? 5 : (inv[IV_STONE_SWORD] ? 3 : (inv[IV_WOOD_SWORD] ? 2 : 1));
                    const int hp = hit_hp - dmg;
#pragma unroll
                    for (int s = 0; s < NSM; ++s)
                        if (l + s * G == hit) { m[s].hp = hp; if (hp <= 0) m[s].alive = 0; }
                    if (hp <= 0) {
                        if (type == MT_ZOMBIE) ach |= 1u << ACH_DEFEAT_ZOMBIE;
                        if (type == MT_SKELETON) ach |= 1u << ACH_DEFEAT_SKELETON;
                        if (type == MT_COW) {
                            vit[1] = min(MAX_COUNT, vit[1] + FOOD_COW);
                            cnt[0] = 0;
                            ach |= 1u << ACH_EAT_COW;
                        }
                    }
                }
            } else {
                int item = -1, leaves = fb, achv = 0;
                bool gate = true;
                switch (fb) {
                case BK_TREE: item = IV_WOOD; achv = ACH_COLLECT_WOOD; break;
                case BK_STONE: item = IV_STONE; gate = inv[IV_WOOD_PICKAXE]; leaves = BK_PATH; achv = ACH_COLLECT_STONE; break;
                case BK_COAL: item = IV_COAL; gate = inv[IV_WOOD_PICKAXE]; leaves = BK_PATH; achv = ACH_COLLECT_COAL; break;
                case BK_IRON: item = IV_IRON; gate = inv[IV_STONE_PICKAXE]; leaves = BK_PATH; achv = ACH_COLLECT_IRON; break;
                case BK_DIAMOND: item = IV_DIAMOND; gate = inv[IV_IRON_PICKAXE]; leaves = BK_PATH; achv = ACH_COLLECT_DIAMOND; break;
                case BK_GRASS: item = IV_SAPLING; gate = sapling_draw < P_SAPLING; achv = ACH_COLLECT_SAPLING; break;
                case BK_WATER:
                    vit[2] = min(MAX_COUNT, vit[2] + 1); cnt[1] = 0; ach |= 1u << ACH_COLLECT_DRINK;
                    break;
                case BK_RIPE:
                    vit[1] = min(MAX_COUNT, vit[1] + FOOD_PLANT); cnt[0] = 0; ach |= 1u << ACH_EAT_PLANT;
                    modval = BK_PLANT;
                    ate_ripe = true;
                    break;
                default: break;
                }
                if (item >= 0 && gate) {
#pragma unroll
                    for (int i = 0; i < 6; ++i)
                        if (i == item && inv[i] < MAX_COUNT) {
                            inv[i]++;
                            ach |= 1u << achv;
                            if (leaves != fb) modval = leaves;
                        }
                }
            }
        }
    } else if (a == AC_SLEEP) {
        if (vit[3] < MAX_COUNT) sleeping = 1;
    } else if (a >= AC_PLACE_STONE && a <= AC_PLACE_PLANT) {
        if (f_in && hit < 0) {
            if (a == AC_PLACE_STONE) {
                if (inv[IV_STONE] >= 1 && (walkable_ground(fb) || fb == BK_WATER || fb == BK_LAVA)) {
                    inv[IV_STONE]--; modval = BK_STONE; ach |= 1u << ACH_PLACE_STONE;
                }
            } else if (a == AC_PLACE_TABLE) {
                if (inv[IV_WOOD] >= 1 && walkable_ground(fb)) {
                    inv[IV_WOOD]--; modval = BK_TABLE; ach |= 1u << ACH_PLACE_TABLE;
                }
            } else if (a == AC_PLACE_FURNACE) {
                if (inv[IV_STONE] >= 1 && walkable_ground(fb) && near_table) {
                    inv[IV_STONE]--; modval = BK_FURNACE; ach |= 1u << ACH_PLACE_FURNACE;
                }
            } else {
                const uint32_t free_slots = ~plant_mask & ((1u << p.cap_plant) - 1u);
                if (inv[IV_SAPLING] >= 1 && fb == BK_GRASS && free_slots) {
                    inv[IV_SAPLING]--; modval = BK_PLANT; ach |= 1u << ACH_PLACE_PLANT;
                    new_plant_slot = __ffs((int)free_slots) - 1;
                }
            }
        }
    } else if (a >= AC_MAKE_WOOD_PICKAXE) {
        const int which = a - AC_MAKE_WOOD_PICKAXE;               // 0..5: pickaxes then swords
        const int tier = which >= 3 ? which - 3 : which;          // 0 wood, 1 stone, 2 iron
        const int need_stone = tier == 1, need_ci = tier == 2;
        const int have = (w_inv >> (24 + which)) & 1;             // tools are made once
        const bool ok = !have && near_table && (!need_ci || near_furnace) && inv[IV_WOOD] >= 1 &&
                        inv[IV_STONE] >= need_stone && inv[IV_COAL] >= need_ci && inv[IV_IRON] >= need_ci;
        if (ok) {
            inv[IV_WOOD]--; inv[IV_STONE] -= need_stone; inv[IV_COAL] -= need_ci; inv[IV_IRON] -= need_ci;
#pragma unroll
            for (int i = 0; i < 6; ++i) if (i == which) inv[6 + i] = 1;
            // achievement ids of the six tools: 5, 13, 20 (pickaxes), 6, 14, 21 (swords)
            const int achv = which >= 3 ? (tier == 0 ? ACH_MAKE_WOOD_SWORD : tier == 1 ? ACH_MAKE_STONE_SWORD : ACH_MAKE_IRON_SWORD)
                                        : (tier == 0 ? ACH_MAKE_WOOD_PICKAXE : tier == 1 ? ACH_MAKE_STONE_PICKAXE : ACH_MAKE_IRON_PICKAXE);
            ach |= 1u << achv;
        }
    }
    const int modcell = modval >= 0 ? fy * MAPW + fx : -1;
    if (modval >= 0) {
        if (l == 0) { map[modcell] = (uint8_t)modval; win[f_win] = (uint8_t)modval; }
#pragma unroll
        for (int s = 0; s < NSP; ++s) {
            const int k = l + s * G;
            if (k == new_plant_slot) { q[s].alive = 1; q[s].x = fx; q[s].y = fy; q[s].age = 0; q_block[s] = BK_PLANT; }
            else if (q[s].alive && q[s].x == fx && q[s].y == fy) { q_block[s] = modval; if (ate_ripe) q[s].age = 0; }
        }
    }
    const int mvx = px - px0, mvy = py - py0;

    // ---- phase 2: mobs.  Intent of each slot from its own state, the player and its draws ----
    int packed[NSM];
    bool l_attack = false, l_arrow_hit = false;
    int n_attack = 0, n_arrow = 0;
#pragma unroll
    for (int s = 0; s < NSM; ++s) {
        const int k = l + s * G;
        int kind = K_NONE, ndir = 0;
        if (m[s].alive) {
            const int type = (k * 11) >> 5;
            const int dx = px - m[s].x, dy = py - m[s].y;
            const int adx = iabs(dx), ady = iabs(dy), cheb = max(adx, ady);
            const uint32_t m8 = dr[s].w[0] >> 29;                 // choice(draw, 8)
            const uint32_t r_act = dr[s].w[1];
            const int toward = adx >= ady ? (dx < 0 ? 1 : 2) : (dy < 0 ? 3 : 4);
            const int wander = m8 < 4 ? (int)m8 + 1 : 0;
            if (type == MT_ZOMBIE) {
                if (m[s].cd > 0) m[s].cd--;
                if (adx + ady == 1) {
                    if (m[s].cd == 0) { kind = K_ATTACK; m[s].cd = CD_ZOMBIE; }
                } else {
                    ndir = (cheb < CHASE_RANGE && r_act < P_CHASE) ? toward : wander;
                    if (ndir) kind = K_MOVE;
                }
            } else if (type == MT_COW) {
                ndir = wander;
                if (ndir) kind = K_MOVE;
            } else if (type == MT_SKELETON) {
                if (m[s].cd > 0) m[s].cd--;
                const bool aligned = (dx == 0 || dy == 0) && cheb <= SHOOT_RANGE;
                if (aligned && m[s].cd == 0 && r_act < P_SHOOT) { kind = K_SHOOT; ndir = toward; m[s].cd = CD_SKELETON; }
                else {
                    ndir = wander ? wander : (cheb <= SHOOT_RANGE ? toward : 0);
                    if (ndir) kind = K_MOVE_PATH;
                }
            } else {
                kind = K_FLY; ndir = m[s].dir;
            }
        }
        const int tx = m[s].x + dir_dx(ndir), ty = m[s].y + dir_dy(ndir);
        const bool t_in = in_map(tx, ty);
        int tb = BK_OOB;
        if (kind != K_NONE && kind != K_ATTACK && t_in) {
            tb = map[ty * MAPW + tx];
            if (ty * MAPW + tx == modcell) tb = modval;
        }
        const bool at_player = (tx == px && ty == py);
        const bool t_ok = t_in && (kind == K_MOVE ? walkable_ground(tb) : (kind == K_MOVE_PATH ? tb == BK_PATH : arrow_flyable(tb)));
        packed[s] = kind | ((int)t_ok << 3) | ((int)at_player << 4) | ((tx + 1) << 8) | ((ty + 1) << 16) | (ndir << 24);
        n_attack += __popc(Gr::ballot(kind == K_ATTACK));
        n_arrow += __popc(Gr::ballot((kind == K_SHOOT || kind == K_FLY) && at_player));
    }
    (void)l_attack; (void)l_arrow_hit;

    // spawn candidates (phase 3) are fixed by the draws and the player's position: read their
    // terrain now so the loads overlap the mob resolution below
    int sp_x[3], sp_y[3], sp_b[3];
    bool sp_cand[3];
    uint32_t sp_p[3];
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        const int dx = (int)choice((uint32_t)Gr::shfl((int)dr[(3 * j) / G].w[3], (3 * j) % G), 31) - 15;
        const int dy = (int)choice((uint32_t)Gr::shfl((int)dr[(3 * j + 1) / G].w[3], (3 * j + 1) % G), 31) - 15;
        sp_p[j] = (uint32_t)Gr::shfl((int)dr[(3 * j + 2) / G].w[3], (3 * j + 2) % G);
        sp_x[j] = px + dx; sp_y[j] = py + dy;
        sp_cand[j] = max(iabs(dx), iabs(dy)) >= SPAWN_MIN_DIST && in_map(sp_x[j], sp_y[j]);
        sp_b[j] = sp_cand[j] ? (int)map[sp_y[j] * MAPW + sp_x[j]] : (int)BK_OOB;
    }

    const int damage = n_attack * (sleeping ? DMG_ZOMBIE_SLEEP : DMG_ZOMBIE) + n_arrow * DMG_ARROW;

    // Moves resolve one slot at a time in the order zombies, cows, arrows, skeletons; each sees
    // the positions left by the slots before it.  An arrow shot now first flies next step.
    constexpr int ORDER[NMOB] = { 0, 1, 2, 3, 4, 5, 9, 10, 11, 6, 7, 8 };
#pragma unroll
    for (int i = 0; i < NMOB; ++i) {
        constexpr int dummy = 0; (void)dummy;
        const int k = ORDER[i];
        const int ks = k / G, kl = k % G;           // owner sub-slot and lane (compile-time)
        const int ik = Gr::shfl(packed[ks], kl);
        const int kk = ik & 7;
        if (Gr::ballot(kk != K_NONE && kk != K_ATTACK) == 0) continue;   // uniform per group
        const bool k_ok = (ik >> 3) & 1, k_at = (ik >> 4) & 1;
        const int kx = ((ik >> 8) & 0xFF) - 1, ky = ((ik >> 16) & 0xFF) - 1;
        bool l_occ = false;
#pragma unroll
        for (int s = 0; s < NSM; ++s) l_occ = l_occ || (m[s].alive && m[s].x == kx && m[s].y == ky);
        const bool occ = Gr::ballot(l_occ) != 0 || (kx == px && ky == py);
        if (kk == K_MOVE || kk == K_MOVE_PATH) {
            if (k_ok && !occ && l == kl) { m[ks].x = kx; m[ks].y = ky; }
        } else if (kk == K_SHOOT) {
            uint32_t arrows = 0;                     // bit j = arrow slot 9+j alive
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const int as = (9 + j) / G, al = (9 + j) % G;
                arrows |= ((Gr::ballot(m[as].alive != 0) >> al) & 1u) << j;
            }
            const uint32_t free_arrows = ~arrows & ((1u << p.cap_arrow) - 1u) & 7u;
            if (!k_at && free_arrows && k_ok && !occ) {
                const int ka = 9 + __ffs((int)free_arrows) - 1;
#pragma unroll
                for (int s = 0; s < NSM; ++s)
                    if (l + s * G == ka) { m[s].alive = 1; m[s].x = kx; m[s].y = ky; m[s].dir = (ik >> 24) & 7; m[s].hp = 0; m[s].cd = 0; }
            }
        } else if (kk == K_FLY) {
            if (l == kl) {
                if (k_at || !k_ok || occ) m[ks].alive = 0;
                else { m[ks].x = kx; m[ks].y = ky; }
            }
        }
    }
    vit[0] = max(0, vit[0] - damage);

    // ---- phase 3: despawn far mobs, then one spawn attempt per type -----------------------------
#pragma unroll
    for (int s = 0; s < NSM; ++s)
        if (m[s].alive && max(iabs(m[s].x - px), iabs(m[s].y - py)) > DESPAWN_DIST) m[s].alive = 0;
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        uint32_t taken = 0;                          // bit i = slot 3j+i alive
        bool l_occ = false;
#pragma unroll
        for (int s = 0; s < NSM; ++s) l_occ = l_occ || (m[s].alive && m[s].x == sp_x[j] && m[s].y == sp_y[j]);
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int ss = (3 * j + i) / G, sl = (3 * j + i) % G;
            taken |= ((Gr::ballot(m[ss].alive != 0) >> sl) & 1u) << i;
        }
        const bool occ = Gr::ballot(l_occ) != 0;
        const uint32_t cap = j == 0 ? p.cap_zombie : (j == 1 ? p.cap_cow : p.cap_skeleton);
        const uint32_t free_slots = ~taken & ((1u << cap) - 1u) & 7u;
        const uint32_t thr = j == 0 ? luts->zombie_thr[phase] : (j == 1 ? P_COW_SPAWN : P_SKELETON_SPAWN);
        const int want = j == 2 ? BK_PATH : BK_GRASS;
        if (sp_cand[j] && free_slots && !occ && sp_b[j] == want && sp_p[j] < thr) {
            const int kn = 3 * j + __ffs((int)free_slots) - 1;
#pragma unroll
            for (int s = 0; s < NSM; ++s)
                if (l + s * G == kn) {
                    m[s].alive = 1; m[s].x = sp_x[j]; m[s].y = sp_y[j]; m[s].dir = 0;
                    m[s].hp = j == 0 ? HP_ZOMBIE : (j == 1 ? HP_COW : HP_SKELETON); m[s].cd = 0;
                }
        }
    }

    // ---- phase 4: plants ----------------------------------------------------------------------------
    if (plant_mask != 0 || new_plant_slot >= 0) {    // uniform per group
        int zinfo[3];
#pragma unroll
        for (int z = 0; z < 3; ++z) {
            const int zs = z / G, zl = z % G;
            zinfo[z] = Gr::shfl((m[zs].alive ? 1 : 0) | (m[zs].x << 8) | (m[zs].y << 16), zl);
        }
#pragma unroll
        for (int s = 0; s < NSP; ++s) {
            if (!q[s].alive) continue;
            bool zombie_near = false;
#pragma unroll
            for (int z = 0; z < 3; ++z)
                zombie_near = zombie_near || ((zinfo[z] & 1) && iabs(((zinfo[z] >> 8) & 0xFF) - q[s].x) + iabs(((zinfo[z] >> 16) & 0xFF) - q[s].y) == 1);
            if (q[s].age < 65535) q[s].age++;
            int nb = q_block[s];
            if (nb == BK_PLANT && q[s].age >= RIPE_AGE) nb = BK_RIPE;
            if (zombie_near && dr[s].w[2] < P_PLANT_EATEN) nb = BK_GRASS;
            if (nb != q_block[s]) {
                map[q[s].y * MAPW + q[s].x] = (uint8_t)nb;
                const int wx = q[s].x - (px0 - WIN_COLS / 2), wy = q[s].y - (py0 - WIN_ROWS / 2);
                if ((unsigned)wx < (unsigned)WIN_COLS && (unsigned)wy < (unsigned)WIN_ROWS) win[wy * WIN_COLS + wx] = (uint8_t)nb;
            }
            if (nb == BK_GRASS) q[s].alive = 0;
        }
    }

    // ---- phase 5: needs ------------------------------------------------------------------------------
    {
        const int asleep = sleeping;
        cnt[0] += asleep ? 1 : 2;
        if (cnt[0] > 50) { cnt[0] = 0; vit[1] = max(0, vit[1] - 1); }
        cnt[1] += asleep ? 1 : 2;
        if (cnt[1] > 40) { cnt[1] = 0; vit[2] = max(0, vit[2] - 1); }
        if (asleep) {
            cnt[2]--;
            if (cnt[2] < -10) { cnt[2] = 0; vit[3] = min(MAX_COUNT, vit[3] + 1); }
        } else {
            cnt[2]++;
            if (cnt[2] > 30) { cnt[2] = 0; vit[3] = max(0, vit[3] - 1); }
        }
        if (vit[0] > 0) {
            const bool fed = vit[1] > 0 && vit[2] > 0 && (vit[3] > 0 || asleep);
            cnt[3] += fed ? (asleep ? 4 : 2) : (asleep ? -1 : -2);
            if (cnt[3] > 50) { cnt[3] = 0; vit[0] = min(MAX_COUNT, vit[0] + 1); }
            if (cnt[3] < -30) { cnt[3] = 0; vit[0]--; }
        }
        if (asleep && (vit[3] >= MAX_COUNT || damage > 0)) { sleeping = 0; ach |= 1u << ACH_WAKE_UP; }
    }

    // ---- reward, time, done ---------------------------------------------------------------------------
    StepOut out;
    out.mvx = mvx; out.mvy = mvy;
    const int gained = __popc(ach & ~ach0);
    out.reward = (float)(10 * gained + (vit[0] - health0)) * 0.1f;
    const uint32_t t1 = t + 1;
    phase = phase + 1 == p.day_length ? 0u : phase + 1;
    out.done = vit[0] <= 0 || t1 >= p.max_episode_steps;
    if (out.done) return out;

    // ---- pack the record back into LDS ------------------------------------------------------------------
    if (l == 0) {
        uint32_t wi = 0;
#pragma unroll
        for (int i = 0; i < 6; ++i) wi |= ((uint32_t)inv[i] << (4 * i)) | ((uint32_t)inv[6 + i] << (24 + i));
        rec[RW_POS] = (uint32_t)px | ((uint32_t)py << 8) | ((uint32_t)dir << 16) | ((uint32_t)sleeping << 24);
        rec[RW_INV] = wi;
        rec[RW_VIT] = (uint32_t)vit[0] | ((uint32_t)vit[1] << 4) | ((uint32_t)vit[2] << 8) | ((uint32_t)vit[3] << 12) | (phase << 16);
        rec[RW_CNT] = (uint32_t)(cnt[0] & 0xFF) | ((uint32_t)(cnt[1] & 0xFF) << 8) | ((uint32_t)(cnt[2] & 0xFF) << 16) | ((uint32_t)(cnt[3] & 0xFF) << 24);
        rec[RW_ACH] = ach;
        rec[RW_T] = t1;
    }
#pragma unroll
    for (int s = 0; s < NSM; ++s) {
        const int k = l + s * G;
        if (k < NMOB) rec[RW_MOB + k] = pack_mob(m[s]);
    }
#pragma unroll
    for (int s = 0; s < NSP; ++s) {
        const int k = l + s * G;
        if (k < NPLANT) rec[RW_PLANT + k] = pack_plant(q[s]);
    }
    group_sync();
    return out;
}

}  // namespace cx
