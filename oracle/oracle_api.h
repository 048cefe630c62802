// CPU ORACLE — TEST INFRASTRUCTURE ONLY.
//
// C prototypes of the oracle's entry points (tuner_oracle.cpp, train_oracle.cpp), for the
// oracle's own translation units and its sanitizer driver.  The Python front end calls the
// same symbols through ctypes.  Nothing of the HIP library includes this file.
#pragma once
#include <stdint.h>

extern "C" {

int oracle_feature_lut(int n_params, const int32_t* radices, const double* values, const int32_t* scales,
                       float* lut_out);
int oracle_digits(int n_params, const int32_t* radices, uint64_t index, int32_t* digits_out);
int oracle_index(int n_params, const int32_t* radices, const int32_t* digits, uint64_t* index_out);
int oracle_predict_range(int n_params, const int32_t* radices, const double* values, const int32_t* scales,
                         int n_constraints, const int32_t* terms, const int64_t* bounds, int n_members,
                         int n_layers, const int32_t* widths, const float* weights, uint64_t begin,
                         uint64_t count, float* yhat, uint8_t* valid, int32_t* digits, int n_threads);
int oracle_predict_indices(int n_params, const int32_t* radices, const double* values, const int32_t* scales,
                           int n_constraints, const int32_t* terms, const int64_t* bounds, int n_members,
                           int n_layers, const int32_t* widths, const float* weights, const uint64_t* indices,
                           uint64_t count, float* yhat, uint8_t* valid, int n_threads);
int64_t oracle_select_topk(const float* yhat, const uint8_t* valid, uint64_t count, uint64_t index_base,
                           int64_t k, float* values_out, uint64_t* indices_out);
int64_t oracle_sample_valid(int n_params, const int32_t* radices, int n_constraints, const int32_t* terms,
                            const int64_t* bounds, uint64_t seed, int64_t n_samples, uint64_t max_draws,
                            uint64_t* indices_out);
int oracle_train_ensemble(int n_params, const int32_t* radices, const double* values, const int32_t* scales,
                          int n_constraints, const int32_t* terms, const int64_t* bounds, int n_members,
                          int hidden, int64_t n_samples, const uint64_t* sample_indices,
                          const float* sample_times, const int32_t* sample_parts, const float* initial_weights,
                          int epochs, float learning_rate, float momentum, float* weights_out, double* loss_out);
double oracle_mean_relative_error(int64_t n, const float* predictions, const float* times, int64_t* n_used);
int64_t oracle_best_of(int64_t m, const float* times, float* best_time);

}  // extern "C"
