// Host side of an adjustment cycle: the policy's forward pass, the choice of an action per
// worker, the batch size update with its clamp, and the reward (paper: Problem Formulation,
// "Reinforcement learning framework", "Action space and batch size adjustment", "Reward function
// design"; Algorithm 1, the action and batch-size steps that follow every k iterations).  The
// policy and value networks are tiny and run on the host once per cycle: plain C++, no device
// work, no allocation beyond two small vectors.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

#include "../../include/dynamix.h"

namespace {
const int32_t kActions[DYNAMIX_NUM_ACTIONS] = {-100, -25, 0, 25, 100};
}

extern "C" {

int64_t dynamix_policy_weight_count(const int32_t* layer_sizes, int32_t num_layers)
{
    if (!layer_sizes || num_layers < 2) return -1;
    int64_t n = 0;
    for (int l = 0; l < num_layers; ++l)
        if (layer_sizes[l] < 1) return -1;
    for (int l = 0; l + 1 < num_layers; ++l)
        n += (int64_t)layer_sizes[l + 1] * layer_sizes[l] + layer_sizes[l + 1];
    return n;
}

int dynamix_policy_forward(const float* weights, const int32_t* layer_sizes, int32_t num_layers,
                           const float* states, int32_t K, float* probs)
{
    if (!weights || !layer_sizes || !states || !probs) return DYNAMIX_ERR_NULL;
    if (K < 1 || dynamix_policy_weight_count(layer_sizes, num_layers) < 0 ||
        layer_sizes[num_layers - 1] != DYNAMIX_NUM_ACTIONS)
        return DYNAMIX_ERR_ARG;
    try {
        int widest = 0;
        for (int l = 0; l < num_layers; ++l) widest = std::max(widest, layer_sizes[l]);
        std::vector<double> cur(widest), nxt(widest);
        for (int k = 0; k < K; ++k) {
            for (int i = 0; i < layer_sizes[0]; ++i) cur[i] = states[(int64_t)k * layer_sizes[0] + i];
            const float* w = weights;   // the same parameters for every worker
            for (int l = 0; l + 1 < num_layers; ++l) {
                const int in = layer_sizes[l], out = layer_sizes[l + 1];
                const float* bias = w + (int64_t)out * in;
                for (int o = 0; o < out; ++o) {
                    double s = bias[o];
                    for (int i = 0; i < in; ++i) s += (double)w[(int64_t)o * in + i] * cur[i];
                    nxt[o] = l + 2 < num_layers ? std::tanh(s) : s;   // the last layer gives logits
                }
                std::swap(cur, nxt);
                w = bias + out;
            }
            double top = cur[0];
            for (int a = 1; a < DYNAMIX_NUM_ACTIONS; ++a) top = std::max(top, cur[a]);
            double e[DYNAMIX_NUM_ACTIONS], z = 0.0;
            for (int a = 0; a < DYNAMIX_NUM_ACTIONS; ++a) z += e[a] = std::exp(cur[a] - top);
            for (int a = 0; a < DYNAMIX_NUM_ACTIONS; ++a)
                probs[(int64_t)k * DYNAMIX_NUM_ACTIONS + a] = (float)(e[a] / z);
        }
    } catch (...) {
        return DYNAMIX_ERR_NOMEM;
    }
    return DYNAMIX_OK;
}

int dynamix_policy_choose(const float* probs, int32_t K, const float* uniforms, int32_t* actions)
{
    if (!probs || !actions) return DYNAMIX_ERR_NULL;
    if (K < 1) return DYNAMIX_ERR_ARG;
    for (int k = 0; k < K; ++k) {
        const float* p = probs + (int64_t)k * DYNAMIX_NUM_ACTIONS;
        int pick = 0;
        if (!uniforms) {   // greedy: the most probable action, the first of equals
            for (int a = 1; a < DYNAMIX_NUM_ACTIONS; ++a)
                if (p[a] > p[pick]) pick = a;
        } else {           // inverse of the cumulative distribution at the caller's uniform draw
            const double u = uniforms[k];
            if (!(u >= 0.0 && u < 1.0)) return DYNAMIX_ERR_ARG;
            double total = 0.0, c = 0.0;
            for (int a = 0; a < DYNAMIX_NUM_ACTIONS; ++a) total += p[a];
            pick = DYNAMIX_NUM_ACTIONS - 1;
            for (int a = 0; a < DYNAMIX_NUM_ACTIONS; ++a) {
                c += p[a];
                if (u * total < c) {
                    pick = a;
                    break;
                }
            }
        }
        actions[k] = pick;
    }
    return DYNAMIX_OK;
}

int dynamix_batch_sizes_step(const int32_t* batch_sizes, const int32_t* actions, int32_t K,
                             int32_t b_min, int32_t b_max, int32_t* next_batch_sizes)
{
    if (!batch_sizes || !actions || !next_batch_sizes) return DYNAMIX_ERR_NULL;
    if (K < 1 || b_min < 1 || b_max < b_min) return DYNAMIX_ERR_ARG;
    for (int k = 0; k < K; ++k)
        if (actions[k] < 0 || actions[k] >= DYNAMIX_NUM_ACTIONS) return DYNAMIX_ERR_ARG;
    for (int k = 0; k < K; ++k) {
        const int64_t moved = (int64_t)batch_sizes[k] + kActions[actions[k]];
        next_batch_sizes[k] = (int32_t)std::max<int64_t>(std::min<int64_t>(moved, b_max), b_min);
    }
    return DYNAMIX_OK;
}

int dynamix_cycle_rewards(const double* mean_accuracy, const double* accuracy_gain,
                          const double* iteration_time, const int32_t* batch_sizes, int32_t K,
                          double alpha, double beta, double delta, double eta, double sigma2_norm,
                          double sigma_norm, int32_t adaptive_optimizer, double* rewards)
{
    if (!mean_accuracy || !accuracy_gain || !iteration_time || !batch_sizes || !rewards)
        return DYNAMIX_ERR_NULL;
    if (K < 1) return DYNAMIX_ERR_ARG;
    for (int k = 0; k < K; ++k)
        if (batch_sizes[k] < 1) return DYNAMIX_ERR_ARG;
    for (int k = 0; k < K; ++k) {
        double r = mean_accuracy[k] + alpha * std::max(0.0, accuracy_gain[k]) - beta * iteration_time[k] -
                   delta * (std::log2((double)batch_sizes[k]) - 5.0);
        if (adaptive_optimizer) r -= eta * (sigma2_norm + sigma_norm);
        rewards[k] = r;
    }
    return DYNAMIX_OK;
}

int dynamix_policy_update(float* weights, const int32_t* layer_sizes, int32_t num_layers,
                          const float* states, const int32_t* actions, const double* signal,
                          const float* old_probs, int64_t n, int32_t mode, double clip_eps, double lr,
                          double* objective)
{
    if (!weights || !layer_sizes || !states || !actions || !signal) return DYNAMIX_ERR_NULL;
    if (mode == DYNAMIX_POLICY_CLIPPED && !old_probs) return DYNAMIX_ERR_NULL;
    const int64_t count = dynamix_policy_weight_count(layer_sizes, num_layers);
    if (n < 1 || count < 0 || layer_sizes[num_layers - 1] != DYNAMIX_NUM_ACTIONS ||
        (mode != DYNAMIX_POLICY_RETURN_WEIGHTED && mode != DYNAMIX_POLICY_CLIPPED) ||
        !(clip_eps >= 0.0) || !(lr == lr))
        return DYNAMIX_ERR_ARG;
    for (int64_t j = 0; j < n; ++j)
        if (actions[j] < 0 || actions[j] >= DYNAMIX_NUM_ACTIONS) return DYNAMIX_ERR_ARG;
    try {
        const int L = num_layers - 1;   // weight layers
        std::vector<double> grad((size_t)count, 0.0);
        std::vector<std::vector<double>> act(num_layers);   // activations of every layer
        for (int l = 0; l < num_layers; ++l) act[l].assign(layer_sizes[l], 0.0);
        std::vector<double> delta, prev;
        double total = 0.0;
        for (int64_t j = 0; j < n; ++j) {
            // forward, keeping the activations
            for (int i = 0; i < layer_sizes[0]; ++i) act[0][i] = states[j * layer_sizes[0] + i];
            const float* w = weights;
            for (int l = 0; l < L; ++l) {
                const int in = layer_sizes[l], out = layer_sizes[l + 1];
                const float* bias = w + (int64_t)out * in;
                for (int o = 0; o < out; ++o) {
                    double s = bias[o];
                    for (int i = 0; i < in; ++i) s += (double)w[(int64_t)o * in + i] * act[l][i];
                    act[l + 1][o] = l + 1 < L ? std::tanh(s) : s;
                }
                w = bias + out;
            }
            const std::vector<double>& z = act[L];
            double top = z[0];
            for (int a = 1; a < DYNAMIX_NUM_ACTIONS; ++a) top = std::max(top, z[a]);
            double p[DYNAMIX_NUM_ACTIONS], zsum = 0.0;
            for (int a = 0; a < DYNAMIX_NUM_ACTIONS; ++a) zsum += p[a] = std::exp(z[a] - top);
            for (int a = 0; a < DYNAMIX_NUM_ACTIONS; ++a) p[a] /= zsum;
            const int aj = actions[j];
            // d(objective_j)/d(logit) = scale * (onehot(a_j) - p)
            double scale;
            if (mode == DYNAMIX_POLICY_RETURN_WEIGHTED) {
                total += signal[j] * std::log(p[aj]);
                scale = signal[j];
            } else {
                const double r = p[aj] / (double)old_probs[j];
                const double clipped = std::min(std::max(r, 1.0 - clip_eps), 1.0 + clip_eps);
                const double plain = r * signal[j], held = clipped * signal[j];
                total += std::min(plain, held);
                // the minimum follows r only where the unclipped term is the smaller one
                scale = plain <= held ? signal[j] * r : 0.0;
            }
            delta.assign(DYNAMIX_NUM_ACTIONS, 0.0);
            for (int a = 0; a < DYNAMIX_NUM_ACTIONS; ++a) delta[a] = scale * ((a == aj ? 1.0 : 0.0) - p[a]);
            // backward through the layers (offsets of layer l's parameters inside the flat vector)
            int64_t end = count;
            for (int l = L - 1; l >= 0; --l) {
                const int in = layer_sizes[l], out = layer_sizes[l + 1];
                const int64_t wofs = end - ((int64_t)out * in + out), bofs = wofs + (int64_t)out * in;
                prev.assign(in, 0.0);
                for (int o = 0; o < out; ++o) {
                    grad[bofs + o] += delta[o];
                    for (int i = 0; i < in; ++i) {
                        grad[wofs + (int64_t)o * in + i] += delta[o] * act[l][i];
                        prev[i] += delta[o] * (double)weights[wofs + (int64_t)o * in + i];
                    }
                }
                if (l > 0)   // through the tanh of layer l's input
                    for (int i = 0; i < in; ++i) prev[i] *= 1.0 - act[l][i] * act[l][i];
                delta.swap(prev);
                end = wofs;
            }
        }
        if (objective) *objective = total / (double)n;
        const double step = lr / (double)n;   // ascent on the mean over the n decisions
        for (int64_t i = 0; i < count; ++i) weights[i] = (float)((double)weights[i] + step * grad[i]);
    } catch (...) {
        return DYNAMIX_ERR_NOMEM;
    }
    return DYNAMIX_OK;
}

double dynamix_discounted_return(const double* rewards, int64_t count, double gamma)
{
    if (!rewards || count < 1) return 0.0;
    double j = 0.0;
    for (int64_t t = count - 1; t >= 0; --t) j = rewards[t] + gamma * j;   // sum_t gamma^t r_t
    return j;
}

}  // extern "C"
