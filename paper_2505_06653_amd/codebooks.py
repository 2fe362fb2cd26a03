"""The 16-level codebooks printed in the paper (appendix "Optimal Quantization Codebooks") and the pin masks.

Level l of the paper (1..16) is index l-1 here.  BOF4 (absolute absmax normalisation) pins {-1, 0, +1} = indices
{0, 7, 15}; BOF4-S (signed absmax) pins {0, +1} = indices {7, 15} (caption of the figure in section 3.1 and the
last paragraph of section 3.2).
"""
import numpy as np
from statistics import NormalDist

PIN_BOF4 = (1 << 0) | (1 << 7) | (1 << 15)
PIN_BOF4S = (1 << 7) | (1 << 15)

# table "Reconstruction levels of BOF4 and BOF4-S optimized w.r.t. MAE and MSE for block size I=64"
BOF4_MAE_64 = (-1.0, -0.7026305794715881, -0.5272703766822815, -0.3946738243103027, -0.2832144796848297,
               -0.1835313588380814, -0.090308666229248, 0.0, 0.0789600014686584, 0.1598792523145676,
               0.244986355304718, 0.3372218906879425, 0.441359281539917, 0.565777063369751, 0.7299178242683411, 1.0)
BOF4_MSE_64 = (-1.0, -0.7535245418548584, -0.579203724861145, -0.4385998845100403, -0.3167679905891418,
               -0.2059924453496933, -0.1015387624502182, 0.0, 0.0887245312333107, 0.1793769598007202,
               0.2741499841213226, 0.3758211433887482, 0.4884937703609467, 0.6187058687210083, 0.7790452241897583,
               1.0)
BOF4S_MAE_64 = (-0.8018798232078552, -0.6076051592826843, -0.468828022480011, -0.3559602797031403,
                -0.2576169371604919, -0.1677481383085251, -0.0827366262674332, 0.0, 0.0789434835314751,
                0.1597966849803925, 0.2448495477437973, 0.3371480107307434, 0.4412573873996735, 0.5656819343566895,
                0.7298068404197693, 1.0)
# table "Reconstruction levels of BOF4-S optimized w.r.t. MSE for various block sizes I"
BOF4S_MSE = {
    32: (-0.8732797503471375, -0.6907446384429932, -0.5437039136886597, -0.4173701703548431, -0.3038933575153351,
         -0.1986017823219299, -0.0981557220220566, 0.0, 0.0925938412547112, 0.187048003077507, 0.2855197489261627,
         0.3907126188278198, 0.506283164024353, 0.6379748582839966, 0.7956376671791077, 1.0),
    64: (-0.8568463921546936, -0.6692874431610107, -0.5235266089439392, -0.4004882574081421, -0.2910638153553009,
         -0.1900092959403992, -0.0938529595732689, 0.0, 0.0887671709060669, 0.1794802695512772, 0.2743096053600311,
         0.3760197460651398, 0.4886530041694641, 0.6188603639602661, 0.7791395783424377, 1.0),
    128: (-0.83739173412323, -0.6462452411651611, -0.5028634667396545, -0.3836247622966766, -0.2783779501914978,
          -0.1815713942050934, -0.0896477326750755, 0.0, 0.0850915610790253, 0.1720834821462631,
          0.2632072865962982, 0.3613293170928955, 0.4707452654838562, 0.5988966822624207, 0.761027991771698, 1.0),
    256: (-0.8146829009056091, -0.6221838593482971, -0.4820549190044403, -0.3669650852680206, -0.2659871876239777,
          -0.1733742356300354, -0.0855776593089104, 0.0, 0.0815095230937004, 0.1649149656295776,
          0.2524392008781433, 0.3470274209976196, 0.4531534314155579, 0.578848659992218, 0.7418596744537354, 1.0),
}


def array(levels):
    return np.array(levels, dtype=np.float64)


def gaussian_quantile_init():
    """Starting codebook for the data-driven Lloyd iterations: 7 negative levels, an exact 0 at index 7 and 8
    positive levels, taken from standard normal quantiles at evenly spaced probabilities on each side and divided
    by the largest so that index 15 is +1.  (A construction of our own in the spirit of quantile-based 4-bit
    codebooks; any sorted start with 0 and +1 in place converges to the same fixed point.)"""
    nd = NormalDist()
    hi = 0.5 + 0.5 * 0.96  # outermost quantile: 96 % of the one-sided mass
    pos = [nd.inv_cdf(0.5 + (hi - 0.5) * k / 8.0) for k in range(1, 9)]
    neg = [-nd.inv_cdf(0.5 + (hi - 0.5) * k / 7.0) for k in range(7, 0, -1)]
    top = pos[-1]
    cb = np.array([v / top for v in neg] + [0.0] + [v / top for v in pos], dtype=np.float64)
    cb[15] = 1.0
    return cb
